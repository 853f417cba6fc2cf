// Prefix-prefill attention over per-request contiguous K/V regions (gfx950, MFMA).
//
// What is computed (paper "Prefix Cache"; "Prefix-prefilling Kernel Evaluation"): new
// token i of request b sits at absolute position P_b + i and attends keys 0 .. P_b + i of
// concat(cached prefix rows, the new tokens' rows): the whole prefix without a mask, the new tokens
// causally.  Prefix rows are read straight from the request's virtually contiguous region (paper
// "vTensor"); the new tokens' rows come from k_new / v_new, or from the region itself when the caller
// has already appended them.
//
// Tiling: a workgroup computes 256 query rows of one (request, kv head) at a time: the G query heads of the
// group for 256/G consecutive new tokens, so one K/V tile read serves every head of the group.  It sweeps the
// visible keys in tiles of 64.  The rows are split over eight wavefronts of 32 rows (head_dim 128: two wavefronts
// per SIMD, 256 registers each) or four wavefronts of 64 rows (one per SIMD, up to 512 registers).  Per tile, with
// v_mfma_f32_32x32x16:
//   S^T[key, row]  = K_tile[64 x D] * Q^T[D x rows of the wavefront]      (A = K from LDS, B = Q in registers)
//   O^T[d, row]   += V_tile^T[D x 64 keys] * P^T[64 keys x rows]         (A = V^T from LDS, B = P in registers)
// Keys run along the rows of S^T, so a softmax reduction over keys is 16 in-lane values plus one
// cross-lane exchange, and the result registers of the first product are, value for value, the B operand
// of the second.
//
// Work distribution: the (item, key tile) pairs of the whole call, items being (request, kv head, token
// tile), form one sequence; workgroup w of n owns the w-th n-th of it.  A workgroup therefore computes some
// whole items and at most two pieces of items it shares with its neighbours.  A whole item is normalised
// and written out at once; a piece leaves its running maxima, sums and unnormalised accumulators in a
// workspace slot, and the workgroup that finishes the last piece of a shared item merges them.  Every
// workgroup gets the same amount of work (in cost units: tiles plus a fixed share per item) whatever the mix of
// lengths, and a call with fewer items than compute units still fills the chip.  Runs of consecutive shares go
// to the same XCD, whose L2 then serves part of the repeated sweeps over one K/V range.
//
// Data movement: K and V tiles go from global memory straight into LDS (global_load_lds, 16 B per lane, no
// registers), four tile buffers, one workgroup barrier per tile.  Both tiles keep their natural [key][d]
// layout; the 16-byte chunks of a row are XOR-swizzled with the row number (applied to the global address,
// since the LDS side of such a load is fixed) so that the MFMA operand reads are bank-conflict free.  The
// V^T operand is read with the transposing LDS read (ds_read_b64_tr_b16): 16 lanes fetch a 4-key x 16-d
// block and each lane receives the 4 keys of its own d.
//
// Softmax: tiles whose 64 keys every row sees ("fast" tiles, swept first) use reference maxima fixed at the start
// of the piece - no maximum tracking, no rescale; an overflow of the weights is detected once per piece and the
// piece redone the classic way.  On the classic path the running maximum is only refreshed when a tile exceeds
// it by more than 2^8, which keeps the accumulator rescale off the common path.  The final division by the
// running sum makes the result independent of which reference maximum was used.
#include <hip/hip_runtime.h>

#include <cmath>
#include <type_traits>

#include "vt_internal.h"

namespace vt {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;

constexpr int kBN = 64;       // keys per tile
constexpr int kRows = 256;    // query rows per workgroup (4 wavefronts x 64)
constexpr float kTau = 8.0f;  // lazy-rescale threshold in log2 units
constexpr int kMinCostPerGroup = 64;  // a workgroup gets at least the work of 32 fast tiles

template <int DT>
struct PElem;
template <>
struct PElem<VT_BF16> {
  static __device__ __forceinline__ f32x16 mfma(u32x4 a, u32x4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0,
                                                   0, 0);
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

// Workgroup i of n runs on XCD i % 8.  Position of workgroup i when the workgroups are listed XCD by XCD (all of
// XCD 0 in launch order, then all of XCD 1, ...): XCD x holds ceil((n - x) / 8) workgroups.
constexpr uint32_t kXcds = 8;
__host__ __device__ inline uint32_t xcd_run_index(uint32_t i, uint32_t n) {
  const uint32_t x = i % kXcds, q = n / kXcds, r = n % kXcds;
  return x * q + (x < r ? x : r) + i / kXcds;
}

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
  float scale_log2e;                   // |scale| * log2(e), at least the smallest normal number
  uint32_t q_sign;                     // 0x80008000 when scale < 0 (the query values are negated instead), else 0
  uint32_t total_cost, n_groups;       // cost units of the whole call, workgroups sharing them
  float* ws;                           // 2 * n_groups piece slots
  unsigned long long* arrivals;        // one word per group: (launch number << 16) | pieces of its shared item done
  unsigned long long launch;           // number of this launch on the context, from 1
};

// Key tiles of item (request with P cached and N new tokens, token tile t of tb tokens).  The keys it sees
// are the P cached rows and the first vis = min((t+1)*tb, N) new rows.  When the new rows come from a buffer
// of their own (split), cached and new rows are tiled separately, so that no tile mixes the two sources.
// A tile is fast when all its 64 keys exist and every query row of the token tile sees them; the others (the
// ragged end of a segment, the causal diagonal) are masked and cost more.
struct ItemShape {
  int nkt, nfast;
};
__host__ __device__ inline ItemShape item_shape(int P, int N, int t, int tb, bool split) {
  const int tok0 = t * tb;
  const int vis = tok0 + tb < N ? tok0 + tb : N;
  const int lenA = split ? P : P + vis, lenB = split ? vis : 0;
  const int seenA = lenA < P + tok0 + 1 ? lenA : P + tok0 + 1;
  ItemShape r;
  r.nkt = (lenA + kBN - 1) / kBN + (lenB + kBN - 1) / kBN;
  r.nfast = seenA / kBN + (split ? (tok0 + 1) / kBN : 0);
  return r;
}
// The work of the call is measured in cost units: a fast tile is kFastCost units, a masked tile kMaskedCost
// (their measured times are about 1.9 and 2.7 microseconds).  Units c .. of an item map to its tiles in sweep
// order (fast tiles first); a tile belongs to whoever owns its first unit: tile_at(c) is the first tile whose
// first unit is >= c.
// An item starts with kItemCost units that belong to no tile: the fixed work of starting and finishing one
// (about 8 microseconds).
constexpr int kFastCost = 2, kMaskedCost = 3, kItemCost = 8;
__host__ __device__ inline uint32_t item_cost(ItemShape s) {
  return (uint32_t)(kItemCost + kFastCost * s.nfast + kMaskedCost * (s.nkt - s.nfast));
}
__host__ __device__ inline int tile_at(ItemShape s, uint32_t c) {
  const int cc = (int)c > kItemCost ? (int)c - kItemCost : 0, cf = kFastCost * s.nfast;
  return cc <= cf ? (cc + kFastCost - 1) / kFastCost : s.nfast + (cc - cf + kMaskedCost - 1) / kMaskedCost;
}
// Cost of all token tiles of one request, per kv head.
__host__ __device__ inline uint32_t request_cost(int P, int N, int tb, bool split) {
  uint32_t c = 0;
  for (int t = 0; t * tb < N; ++t) c += item_cost(item_shape(P, N, t, tb, split));
  return c;
}
// First cost unit of workgroup w.
__host__ __device__ inline uint32_t group_begin(uint32_t total, uint32_t n, uint32_t w) {
  return (uint32_t)((uint64_t)total * w / n);
}
// Floats of one piece slot: 256 maxima, 256 sums, 256 x D accumulators.
__host__ __device__ constexpr uint32_t piece_floats(int d) { return 512u + 256u * (uint32_t)d; }
// 16 bytes per lane from global memory straight into LDS: lane l lands at LDS address lds_base + LDS_OFF + 16*l
// (lds_base uniform) and fetches from base + row_off + (chunk ^ XOR) (base uniform, the rest 32-bit lane values).
// Written as assembly so that these loads are invisible to the compiler's wait-count bookkeeping: it would
// otherwise guard operand reads of the tile buffers with waits for every outstanding load.  The kernel places
// its own waits (wait_loads) and barriers.  m0 (the LDS address; nothing else in this file uses it) must be
// written one instruction before the load reads it: the lane offset is worked out in between.
template <int LDS_OFF, int XOR>
__device__ __forceinline__ void dma16(const char* base, uint32_t row_off, uint32_t chunk, uint32_t lds_base) {
  static_assert(XOR >= 0 && XOR <= 64, "inline constant");
  uint32_t t;
  asm volatile("s_add_u32 m0, %3, %4\n\tv_xad_u32 %0, %1, %5, %2\n\tglobal_load_lds_dwordx4 %0, %6"
               : "=&v"(t)
               : "v"(chunk), "v"(row_off), "s"(lds_base), "n"(LDS_OFF), "n"(XOR), "s"(base)
               : "memory", "scc");
}
// Accesses at device scope for data that workgroups on different XCDs hand to each other inside one launch (each
// XCD has its own L2): the store goes through to memory, the load does not take the line from this XCD's L2.
// Written as assembly so that they come 16 bytes wide; the caller waits (wait_device_accesses) before it relies on a
// store having landed or uses a loaded value.
__device__ __forceinline__ void store16_device(float* p, f32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" : : "v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void load16_device(f32x4& v, const float* p) {
  asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(v) : "v"(p) : "memory");
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

// Where cost unit `cursor` of the whole sequence lies: item (b, g, t), unit c of it.  Items are ordered by
// request, kv head, token tile.  s_pre[b] = cost of the requests before b (all heads).  Every value is the same
// in all lanes.
struct ItemPos {
  int b, g, t;
  uint32_t c;
  ItemShape shape;
};
__device__ __forceinline__ int find_request(const PrefillParams& p, const uint32_t* s_pre, uint32_t cursor) {
  int lo = 0, hi = (int)p.batch;  // last b with s_pre[b] <= cursor
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if ((uint32_t)uni((int)s_pre[mid]) <= cursor) lo = mid; else hi = mid;
  }
  return lo;
}
// P and N of the request come from the caller (who may have them at hand).
__device__ __forceinline__ ItemPos locate(const PrefillParams& p, const uint32_t* s_pre, uint32_t cursor, bool split,
                                          int lo, int P, int N) {
  ItemPos r;
  r.b = lo;
  const uint32_t first = (uint32_t)uni((int)s_pre[lo]);
  const uint32_t per_head = ((uint32_t)uni((int)s_pre[lo + 1]) - first) / p.hkv;
  const uint32_t local = cursor - first;
  r.g = (int)(local / per_head);
  uint32_t rem = local - (uint32_t)r.g * per_head;
  int t = 0;
  ItemShape sh = item_shape(P, N, 0, (int)p.tb, split);
  while (rem >= item_cost(sh) && (t + 1) * (int)p.tb < N) {
    rem -= item_cost(sh);
    ++t;
    sh = item_shape(P, N, t, (int)p.tb, split);
  }
  r.t = t;
  r.c = rem;
  r.shape = sh;
  return r;
}
__device__ __forceinline__ void build_prefix(const PrefillParams& p, uint32_t* s_pre, int tid, int n_threads,
                                             bool split) {
  const int B = (int)p.batch;
  for (int r = tid; r < B; r += n_threads)
    s_pre[r + 1] = request_cost(p.plens[r], p.cu[r + 1] - p.cu[r], (int)p.tb, split) * p.hkv;
  __syncthreads();
  if (tid == 0) {
    uint32_t run = 0;
    s_pre[0] = 0;
    for (int r = 1; r <= B; ++r) {
      run += s_pre[r];
      s_pre[r] = run;
    }
  }
  __syncthreads();
}

// One contiguous run of an item's tiles, computed by this workgroup.  Every field is the same in all lanes.
struct Tile {
  const char* k;
  const char* v;
  int last_row;  // rows 0 .. last_row exist
  int jbase;     // absolute position of the key in row 0
};
struct Piece {
  int valid;
  int b, g, t;            // the item: request, kv head, token tile
  int P, N, cu_b;         // cached rows, new rows, first new row of the request
  int s0, s1;             // tiles [s0, s1) of the item's sweep
  int nkt, nfast;         // tiles and fast tiles of the whole item
  uint32_t item_begin;    // first cost unit of the item in the whole sequence
  uint32_t end_pos;       // cost unit after the piece: the end of its item, or the end of the workgroup's range
  int lenA, lenB, nA, fastA, fastB;
  const char *kc, *vc, *kn, *vn;  // row 0 of segment A (region) and of segment B (k_new / v_new), at this kv head
};

// RB: 32-row blocks of query rows per wavefront.  RB = 2: four wavefronts of 64 rows, one per SIMD, each with up to 512
// registers per lane.  RB = 1: eight wavefronts of 32 rows, two per SIMD with 256 registers each - every K and V operand
// read then feeds one MFMA instead of two (twice the LDS traffic), but while one wavefront of a SIMD waits for LDS or
// works on its weights the other one's MFMAs run.
template <int DT, int D, int RB>
__global__ __launch_bounds__(64 * (8 / RB)) void prefill_kernel(PrefillParams p) {
  constexpr int NW = 8 / RB;           // wavefronts
  constexpr int NT = 64 * NW;          // threads
  constexpr int WR = 32 * RB;          // query rows per wavefront
  constexpr int CH = D / 8;            // 16-byte chunks per head row
  constexpr int KS = D / 16;           // k-steps of the score product
  constexpr int DB = D / 32;           // 32-row d blocks of the value product
  constexpr int ROWB = D * 2;          // bytes per head row
  constexpr int RPL = 256 / ROWB;      // rows per 256-byte LDS bank line
  constexpr int RPI = 64 / CH;         // rows filled by one wavefront-wide load
  constexpr int TILEB = kBN * ROWB;    // bytes of one K (or V) tile
  constexpr int NLD = kBN / RPI / NW;  // loads per wavefront, tile and tensor
  constexpr int STG = 64 + 16;         // bytes of one output staging row: 32 values and a pad
  // Four tile buffers (K tile, then V tile each).
  __shared__ __attribute__((aligned(1024))) char lds_tiles[4 * 2 * TILEB];
  // Output staging, one area per wavefront (the tile buffers are never free: the next piece's tiles are on their way).
  __shared__ __attribute__((aligned(16))) char lds_stage[NW][WR * STG];
  __shared__ uint32_t s_pre[kMaxPrefillBatch + 1];
  // Lengths and region addresses of the first few requests this workgroup works on, fetched once: a piece then
  // starts without a round trip to memory for them.
  constexpr int kWin = 8;
  __shared__ int s_wP[kWin], s_wN[kWin], s_wCu[kWin];
  __shared__ const char* s_wK[kWin];
  __shared__ const char* s_wV[kWin];
  // Per wavefront: the three tiles that follow the current piece in this workgroup's tile stream (address of K row
  // 0, of V row 0, last row), written when the piece starts and read when the loads run past its end.
  __shared__ int s_ahead[NW][3][6];
  __shared__ int s_vote[NW];
  __shared__ unsigned s_arrived;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int col = lane & 31, hi = lane >> 5;
  const int G = (int)p.group, tb = (int)p.tb;
  const bool split_src = p.k_new != nullptr;
  const uint32_t row_bytes = p.hkv * D * 2;

  build_prefix(p, s_pre, tid, NT, split_src);
  // Which group of the plan this workgroup is.  Workgroups are handed to the 8 XCDs in turn (workgroup i runs on
  // XCD i mod 8), and neighbouring groups sweep the same K/V rows (consecutive token tiles of one request and KV
  // head) at about the same time: give each XCD a run of consecutive groups, so that its L2 serves the re-reads.
  const uint32_t group = xcd_run_index(blockIdx.x, p.n_groups);
  uint32_t cursor = group_begin(p.total_cost, p.n_groups, group);
  const uint32_t range_end = group_begin(p.total_cost, p.n_groups, group + 1);
  const int b_win = cursor < range_end ? find_request(p, s_pre, cursor) : 0;
  if (tid < kWin && b_win + tid < (int)p.batch) {
    const int r = b_win + tid;
    s_wP[tid] = p.plens[r];
    s_wCu[tid] = p.cu[r];
    s_wN[tid] = p.cu[r + 1] - p.cu[r];
    s_wK[tid] = p.k_ptrs[r];
    s_wV[tid] = p.v_ptrs[r];
  }
  __syncthreads();

  // Fills in the fields of a piece that follow from its item (b, g, t), the request's lengths and its tile range.
  auto finish_piece = [&](Piece& r, const char* k_req, const char* v_req) {
    const int tok0 = r.t * tb;
    const int vis = min(tok0 + tb, r.N);          // new rows the last token of the tile sees
    // Two key segments: A = rows of the region (the cached prefix; also the new rows when they are already in
    // the cache), B = rows of k_new / v_new.  Each is tiled from its own row 0.
    r.lenA = split_src ? r.P : r.P + vis;
    r.lenB = split_src ? vis : 0;
    r.nA = (r.lenA + kBN - 1) / kBN;
    // Tiles whose 64 keys every row of the workgroup sees: inside a segment and not beyond the first token.
    r.fastA = min(r.lenA, r.P + tok0 + 1) / kBN;
    r.fastB = split_src ? (tok0 + 1) / kBN : 0;
    r.kc = k_req + (size_t)r.g * ROWB;
    r.vc = v_req + (size_t)r.g * ROWB;
    r.kn = split_src ? uni(p.k_new + (size_t)r.cu_b * row_bytes + (size_t)r.g * ROWB) : r.kc;
    r.vn = split_src ? uni(p.v_new + (size_t)r.cu_b * row_bytes + (size_t)r.g * ROWB) : r.vc;
  };
  // Lengths and region bases of request b (from the window when it is there).
  struct Req {
    int P, N, cu_b;
    const char *k, *v;
  };
  auto request = [&](int b) -> Req {
    const bool in_win = b - b_win < kWin;
    const int wi = in_win ? b - b_win : 0;
    Req q;
    q.cu_b = uni(in_win ? s_wCu[wi] : p.cu[b]);
    q.P = uni(in_win ? s_wP[wi] : p.plens[b]);
    q.N = uni(in_win ? s_wN[wi] : p.cu[b + 1] - p.cu[b]);
    q.k = uni(in_win ? s_wK[wi] : p.k_ptrs[b]);
    q.v = uni(in_win ? s_wV[wi] : p.v_ptrs[b]);
    return q;
  };
  // The first piece of this workgroup's range: the tiles of an item whose first cost unit lies in the range
  // (valid = 0 when the range holds none).  A search in the table of request costs; later pieces follow from
  // their predecessor (next_piece).
  auto first_piece = [&](uint32_t pos) -> Piece {
    Piece r;
    r.valid = 0;
    while (pos < range_end) {
      const int b = find_request(p, s_pre, pos);
      const Req q = request(b);
      const ItemPos ip = locate(p, s_pre, pos, split_src, b, q.P, q.N);
      const uint32_t cost = item_cost(ip.shape);
      const uint32_t c1 = min(cost, ip.c + (range_end - pos));
      const int s0 = tile_at(ip.shape, ip.c), s1 = tile_at(ip.shape, c1);
      const uint32_t item_begin = pos - ip.c;
      pos += c1 - ip.c;
      if (s1 <= s0) continue;
      r.valid = 1;
      r.b = b;
      r.g = ip.g;
      r.t = ip.t;
      r.P = q.P;
      r.N = q.N;
      r.cu_b = q.cu_b;
      r.s0 = s0;
      r.s1 = s1;
      r.nkt = ip.shape.nkt;
      r.nfast = ip.shape.nfast;
      r.item_begin = item_begin;
      r.end_pos = pos;
      finish_piece(r, q.k, q.v);
      return r;
    }
    return r;
  };
  // The piece after `pc` in this workgroup's range.  When pc stops at the end of the range there is none; otherwise
  // pc ran to the end of its item and the next item starts where it ended: the next token tile of the same request
  // and kv head, else the next kv head, else the next request that has new tokens.
  auto next_piece = [&](const Piece& pc) -> Piece {
    Piece r = pc;
    r.valid = 0;
    if (pc.end_pos >= range_end) return r;
    const char* k_req = pc.kc - (size_t)pc.g * ROWB;
    const char* v_req = pc.vc - (size_t)pc.g * ROWB;
    r.t = pc.t + 1;
    if (r.t * tb >= pc.N) {
      r.t = 0;
      r.g = pc.g + 1;
      if (r.g == (int)p.hkv) {
        r.g = 0;
        Req q;
        q.N = 0;
        int b = pc.b;
        while (q.N == 0) {
          if (++b >= (int)p.batch) return r;  // (cannot happen: the range ends with the last item)
          q = request(b);
        }
        r.b = b;
        r.P = q.P;
        r.N = q.N;
        r.cu_b = q.cu_b;
        k_req = q.k;
        v_req = q.v;
      }
    }
    const ItemShape sh = item_shape(r.P, r.N, r.t, tb, split_src);
    const uint32_t c1 = min(item_cost(sh), range_end - pc.end_pos);
    r.item_begin = pc.end_pos;
    r.end_pos = pc.end_pos + c1;
    r.s0 = 0;
    r.s1 = tile_at(sh, c1);
    r.nkt = sh.nkt;
    r.nfast = sh.nfast;
    if (r.s1 <= 0) return r;  // the range ends before the item's first tile
    r.valid = 1;
    finish_piece(r, k_req, v_req);
    return r;
  };
  // An item's tiles are swept in this order: the fast tiles of A, the fast tiles of B, then the rest of A (its
  // ragged last tile) and the rest of B (the causal diagonal).  Softmax does not care about the order of the
  // keys, and this way the unmasked tiles come first.  Tile s of the sweep of piece pc's item:
  auto tile_in = [&](const Piece& pc, int s) -> Tile {
    // (bitwise operators on purpose: plain scalar selects, no branches in the middle of the tile code)
    const int nfast_item = pc.fastA + pc.fastB;
    const bool in_b = ((s >= pc.fastA) & (s < nfast_item)) | (s >= nfast_item + pc.nA - pc.fastA);
    const int tt = s - (s < pc.fastA ? 0 : (s < nfast_item ? pc.fastA : (in_b ? pc.nA : pc.fastB)));
    Tile r;
    const size_t off = (size_t)tt * kBN * row_bytes;
    r.k = (in_b ? pc.kn : pc.kc) + off;
    r.v = (in_b ? pc.vn : pc.vc) + off;
    r.last_row = min(kBN, (in_b ? pc.lenB : pc.lenA) - tt * kBN) - 1;
    r.jbase = (in_b ? pc.P : 0) + tt * kBN;
    return r;
  };

  // The piece being computed.  (Plain variables rather than the struct in the lambdas below: the tile code refers
  // to a handful of them only.)
  Piece cur = first_piece(cursor);
  if (!cur.valid) return;
  int s0, s1, P, ntok;
  auto tile_of = [&](int s) -> Tile { return tile_in(cur, s); };
  // Descriptor for a tile that is loaded ahead of its use.  The workgroup's pieces form one stream of tiles and the
  // loads run three tiles ahead of the arithmetic right through the piece boundaries: past the end of the piece
  // they fetch the first tiles of the next pieces (looked up once per piece and parked in LDS, see park_ahead).
  // Past the end of the stream the loads go on as well (so that the count of outstanding loads, and with it the
  // wait at every tile, stays the same), into buffers nobody reads: every lane then fetches from row 0 of the last
  // tile - a few cache lines instead of a tile.
  auto tile_ahead = [&](int s) -> Tile {
    if (__builtin_expect(s < s1, 1)) return tile_of(s);
    asm volatile("" ::: "memory");  // a real branch: the look-up is not to be hoisted above the test
    const int* a = s_ahead[wave][s - s1];
    Tile r;
    const uint32_t klo = (uint32_t)uni(a[0]), khi = (uint32_t)uni(a[1]);
    const uint32_t vlo = (uint32_t)uni(a[2]), vhi = (uint32_t)uni(a[3]);
    r.k = (const char*)(((uint64_t)khi << 32) | klo);
    r.v = (const char*)(((uint64_t)vhi << 32) | vlo);
    r.last_row = uni(a[4]);
    r.jbase = 0;
    return r;
  };
  // End of the run of fast tiles of one segment that holds tile s of the current piece (s + 1 when s is not such a
  // tile): up to there, each tile lies 64 rows after its predecessor.
  auto run_end_of = [&](int s) -> int {
    const int nfast_item = cur.fastA + cur.fastB;
    return s < cur.fastA ? min(cur.fastA, s1) : (s < min(nfast_item, s1) ? min(nfast_item, s1) : s + 1);
  };
  // Looks up the three tiles that follow the current piece in the stream and parks them.
  auto park_ahead = [&]() {
    Piece nx = next_piece(cur);
    int s = 0;
    Tile last = tile_of(s1 - 1);
    last.last_row = 0;
#pragma unroll 1
    for (int j = 0; j < 3; ++j) {
      if (nx.valid && s >= nx.s1) {
        nx = next_piece(nx);
        s = 0;
      }
      Tile tl = last;
      if (nx.valid) {
        tl = tile_in(nx, s++);
        last = tl;
        last.last_row = 0;
      }
      int* a = s_ahead[wave][j];
      a[0] = (int)(uint32_t)(uint64_t)tl.k;
      a[1] = (int)(uint32_t)((uint64_t)tl.k >> 32);
      a[2] = (int)(uint32_t)(uint64_t)tl.v;
      a[3] = (int)(uint32_t)((uint64_t)tl.v >> 32);
      a[4] = tl.last_row;
    }
  };

  // Query rows of this lane (one per 32-column block): the G heads of the group for consecutive tokens.  Rows past
  // the last token of the tile are padding: zeros (their scores and weights are then constants, the cheapest
  // operands to multiply), never written.  A negative scale is applied as |scale| to scores of the negated queries:
  // the kernel takes maxima of raw scores and multiplies afterwards, which needs a non-negative factor.
  auto load_q = [&](const Piece& pc, u32x4 (*q)[KS]) {
    const int tok0 = pc.t * tb, nt = min(tb, pc.N - tok0);
#pragma unroll
    for (int cb = 0; cb < RB; ++cb) {
      const int r = wave * WR + cb * 32 + col;
      const int t = r / G, q_head = r - t * G;
      const int q_tok = min(t, nt - 1);
      const unsigned keep = t < nt ? 0xffffffffu : 0u;
      const char* qp = p.q + ((size_t)(pc.cu_b + tok0 + q_tok) * p.hq + (size_t)pc.g * G + q_head) * ROWB;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const u32x4 raw = *(const u32x4*)(qp + (16 * ks + 8 * hi) * 2);
        q[cb][ks] = u32x4{(raw[0] ^ p.q_sign) & keep, (raw[1] ^ p.q_sign) & keep, (raw[2] ^ p.q_sign) & keep,
                          (raw[3] ^ p.q_sign) & keep};
      }
    }
  };
  int lim[RB];
  int run_end = 0;  // end of the run of fast tiles (see run_end_of) that holds the tile the fast-tile code loads next
  u32x4 qf[RB][KS];
  f32x16 acc[DB][RB];
  float m_used[RB], l_run[RB];
  bool wave_idle;
  load_q(cur, qf);

  // Tile loads.  Load i of this wavefront fills LDS rows (NLD*wave + i)*RPI .. +RPI-1 of the tile; the lane
  // lands in row `row` at chunk position ld_pos and therefore fetches the chunk that the swizzle assigns to
  // that position.  K rows are swizzled with (row/RPL) % CH, V rows with 4*((row/RPL) % (CH/4)).  Rows past the
  // end of the segment repeat its last row (they are masked later).  A tile's loads are issued a pair (one of
  // K, one of V) at a time between the compute stages rather than back to back.  A few values per lane stay in
  // registers: the byte offset of its row in every load and its swizzled chunk offsets in load 0.  Load i is RPI*i rows
  // further; RPI/RPL is 4 and the lane's row/RPL in load 0 is below 4 modulo 4*NLD, so the K swizzle of load i is
  // that of load 0 with 4*i XORed in (64*i in bytes) and the V swizzle does not depend on i.  A tile buffer is the K
  // tile followed by the V tile.
  static_assert(RPI / RPL == 4 && 64 / CH / RPL == 4 && (4 * NLD) <= CH, "swizzle of load i from that of load 0");
  const int ld_r = wave * NLD * RPI + lane / CH, ld_pos = lane % CH;
  uint32_t ld_row[NLD];  // byte offset of the lane's row in load i
#pragma unroll
  for (int i = 0; i < NLD; ++i) ld_row[i] = (uint32_t)(ld_r + i * RPI) * row_bytes;
  const uint32_t ld_chunk_k = (uint32_t)((ld_pos ^ ((ld_r / RPL) % CH)) * 16);
  const uint32_t ld_chunk_k2 = ld_chunk_k ^ 128u;  // (loads 2 and 3: XORs with 128 and 192 = 128 ^ 64)
  const uint32_t ld_chunk_v = (uint32_t)((ld_pos ^ (4 * ((ld_r / RPL) % (CH / 4)))) * 16);
  auto issue_part = [&](auto part, const Tile& tl, char* tile_k) {
    constexpr int i = decltype(part)::value;
    const uint32_t lb = (uint32_t)uni((int)lds_addr_of(tile_k) + wave * NLD * 1024);
    const uint32_t row_i = ld_row[i < NLD ? i : 0], row_last = __umul24((unsigned)tl.last_row, row_bytes);
    const uint32_t ro = row_i < row_last ? row_i : row_last;
    dma16<i * 1024, (i & 1) * 64>(tl.k, ro, i < 2 ? ld_chunk_k : ld_chunk_k2, lb);
    dma16<TILEB + i * 1024, 0>(tl.v, ro, ld_chunk_v, lb);
  };
  static_assert(NLD == 2 || NLD == 4, "tile load split");
  const std::integral_constant<int, 0> part0;
  const std::integral_constant<int, 1> part1;
  const std::integral_constant<int, 2> part2;
  const std::integral_constant<int, 3> part3;
  auto issue_tile = [&](const Tile& tl, char* tile_k) {
    issue_part(part0, tl, tile_k);
    issue_part(part1, tl, tile_k);
    if constexpr (NLD > 2) {
      issue_part(part2, tl, tile_k);
      issue_part(part3, tl, tile_k);
    }
  };

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

  // In a run of fast tiles the K operand reads go through one LDS address per k-step that follows the tile buffers:
  // k_at[ks] is the lane's address for key block 0 of the current tile (block 1 is a constant further).
  uint32_t k_at[KS];
  auto lds_read16 = [](uint32_t addr) -> u32x4 {
    return *(const __attribute__((address_space(3))) u32x4*)addr;
  };
  auto read_k = [&](auto ksc, const char* tk, int kb) -> u32x4 {
    constexpr int ks = decltype(ksc)::value;
    return *(const u32x4*)(tk + (32 * kb + col) * ROWB + (((2 * ks + hi) ^ kswz) * 16));
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
  // MFMA i of the value product of one 32-key block: operand i/RB, query column block i%RB.
  constexpr int NVR = 4 * DB;       // transposing reads of one V block
  constexpr int NPV = 2 * DB * RB;  // MFMAs of one value product
  auto pv_mfma = [&](auto ic, const u32x2* vh, u32x4 (*pf)[2]) {
    constexpr int i = decltype(ic)::value;
    constexpr int m = i / RB, cb = i % RB, db = m / 2, s2 = m % 2;
    u32x4 f;
    f[0] = vh[2 * m][0];
    f[1] = vh[2 * m][1];
    f[2] = vh[2 * m + 1][0];
    f[3] = vh[2 * m + 1][1];
    acc[db][cb] = PElem<DT>::mfma(f, pf[cb][s2], acc[db][cb]);
  };
  auto zero = [](f32x16& x) {
#pragma unroll
    for (int i = 0; i < 16; ++i) x[i] = 0.f;
  };
  // S^T block (32 keys x the wavefront's rows) = K Q^T.
  auto scores = [&](const char* tk, int kb, f32x16* s) {
#pragma unroll
    for (int cb = 0; cb < RB; ++cb) zero(s[cb]);
    static_for<0, KS>([&](auto ks) {
      const u32x4 kf = read_k(ks, tk, kb);
#pragma unroll
      for (int cb = 0; cb < RB; ++cb) s[cb] = PElem<DT>::mfma(kf, qf[cb][ks], s[cb]);
    });
  };
  // One of the nine steps that turn a 32-key x 32-row score block (16 values per lane) into softmax weights
  // against the current reference maximum: step j < 8 computes weights 2j and 2j+1, step j >= 1 rounds the
  // previous pair to the storage type (they are the MFMA operand), stores it as word j-1 of the operand and
  // adds it to the partial sum.  The sum is taken over the rounded weights, two per instruction (dot product
  // of the packed pair with ones): the normaliser then matches the numerator exactly.
  // With a mask, value e of the block (key row 8*(e/4) + e%4 past the lane's first row) only counts when that
  // offset does not exceed thr.
  auto weight_step = [&](auto jc, const f32x16& sv, float nm, float* pr, u32x4* pw, float& ps, auto masked,
                         int thr) {
    constexpr int j = decltype(jc)::value;
    if constexpr (j < 8) {
      pr[2 * j] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[2 * j], c, nm));
      pr[2 * j + 1] = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[2 * j + 1], c, nm));
      if constexpr (decltype(masked)::value) {
        constexpr int e0 = 2 * j, e1 = 2 * j + 1;
        pr[e0] = 8 * (e0 / 4) + e0 % 4 <= thr ? pr[e0] : 0.f;
        pr[e1] = 8 * (e1 / 4) + e1 % 4 <= thr ? pr[e1] : 0.f;
      }
    }
    if constexpr (j >= 1) {
      const unsigned w = PElem<DT>::pack2(pr[2 * j - 2], pr[2 * j - 1]);
      pw[(j - 1) / 4][(j - 1) % 4] = w;
      ps = PElem<DT>::add_pair(w, ps);
    }
  };
  auto weights = [&](const f32x16* s, u32x4 (*pf)[2]) {
#pragma unroll
    for (int cb = 0; cb < RB; ++cb) {
      float pr[16], ps = 0.f;
      // (a row that has seen no key yet - possible when a piece starts on the causal diagonal - has no maximum;
      // its scores are all -inf and must give weight 0, not exp2(-inf + inf))
      const float nm = m_used[cb] == -INFINITY ? 0.f : -m_used[cb];
      static_for<0, 9>([&](auto j) { weight_step(j, s[cb], nm, pr, pf[cb], ps, std::false_type{}, 0); });
      l_run[cb] += ps;
    }
  };
  // Column maxima of a score block (over the lane's 16 keys and its partner half), in exp2 units.
  auto block_max = [&](const f32x16* s, float* tmax) {
#pragma unroll
    for (int cb = 0; cb < RB; ++cb) {
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
  // Tile pipeline.  The workgroup's tiles form one stream; the tile at stream position i lives in buffer i % 4.
  // While tile kt is computed, tiles kt+1
  // and kt+2 are in flight or landed.  Every tile kt follows the same protocol.  Before its synchronisation
  // point it issues loads 1 and 2 of tile kt+2 (only load 1 when a tile has two loads per tensor).  At the
  // synchronisation point the wavefront waits until its own part of tile kt+1 has landed - loads complete in
  // order, so it waits until at most the SYNC_N loads issued after that tile's last one are outstanding -
  // then, past the barrier, everyone's part has landed and everyone is done with tile kt-1.  After it, it
  // issues the last load of tile kt+2 (when there are four) and load 0 of tile kt+3, which goes into the
  // buffer of tile kt-1.  Past the last tile the refills go on as dummies (see tile_ahead), which keeps the count
  // of outstanding loads, and with it the wait, the same on every tile.  The barrier is the
  // bare instruction: the fence of __syncthreads would wait for all outstanding loads.
  constexpr int SYNC_N = NLD > 2 ? VM - 2 : VM;
  auto sync_next = [&]() {
    wait_loads(std::integral_constant<int, SYNC_N>{});
    __builtin_amdgcn_s_barrier();
  };
  auto issue_before_sync = [&](const Tile& t2, char* gk) {
    issue_part(part1, t2, gk);
    if constexpr (NLD > 2) issue_part(part2, t2, gk);
  };
  auto issue_after_sync = [&](const Tile& t2, const Tile& t3, char* gk, char* fk) {
    if constexpr (NLD > 2) issue_part(part3, t2, gk);
    issue_part(part0, t3, fk);
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
  // ck: this tile's buffer (K, then V); nk: the next tile's; gk: buffer of tile kt+2; fk: buffer of tile kt+3.
  // k0 holds K block 0 of this tile on entry and of the next tile on exit; t2 describes tile kt+2 on entry and
  // tile kt+3 (the next tile's kt+2) on exit.
  static_assert(RB == 1 || NPV == 2 * KS, "V reads are spread one per slot over two score stages");
  auto fast_tile = [&](auto masked, int kt, const char* ck, const char* nk, char* gk, char* fk, u32x4* k0, Tile& t2) {
    if constexpr (RB == 2) {
      f32x16 s0v[2], s1v[2];
      u32x4 p0[2][2], p1[2][2];
      u32x4 k1[KS];
      u32x2 v0h[NPV], v1h[NPV];
      float pr[16];
      const float nm0 = -m_used[0], nm1 = -m_used[1];
      const char* cv = ck + TILEB;
      const uint32_t k_step = (uint32_t)uni((int)(lds_addr_of(nk) - lds_addr_of(ck)));
      // masked variant: rows of the tile the two query rows of the lane see, as offsets from the lane's first row
      // of key block 0 (block 1 is 32 further)
      int thr0 = 0, thr1 = 0;
      if constexpr (decltype(masked)::value) {
        const Tile cur = tile_of(kt);
        thr0 = min(lim[0] - cur.jbase, cur.last_row) - 4 * hi;
        thr1 = min(lim[1] - cur.jbase, cur.last_row) - 4 * hi;
      }
      // Tile kt+3.  Inside a run of fast tiles of one segment it is 64 rows after tile kt+2; a full look-up otherwise.
      // (Here rather than where stage F uses it: the look-up branches, and with a branch between them the compiler
      // moves the weights of stages D and E down to their first use in F, off the slots they were given.)
      Tile t3;
      if (__builtin_expect(kt + 3 < run_end, 1)) {
        t3.k = t2.k + (size_t)kBN * row_bytes;
        t3.v = t2.v + (size_t)kBN * row_bytes;
        t3.last_row = kBN - 1;
        t3.jbase = 0;
      } else {
        t3 = tile_ahead(kt + 3);
        run_end = run_end_of(kt + 3);
      }
      // A
      zero(s0v[0]);
      static_for<0, KS>([&](auto i) {
        s0v[0] = PElem<DT>::mfma(k0[i], qf[0][i], s0v[0]);
        k1[i] = lds_read16(k_at[i] + 32 * ROWB);
        if constexpr (i == 0) issue_part(part1, t2, gk);
        if constexpr (i == KS / 2 && NLD > 2) issue_part(part2, t2, gk);
        __builtin_amdgcn_sched_barrier(0);
      });
      // B
      zero(s0v[1]);
      static_for<0, KS>([&](auto i) {
        s0v[1] = PElem<DT>::mfma(k0[i], qf[1][i], s0v[1]);
        static_for<i * 9 / KS, (i + 1) * 9 / KS>([&](auto j) { weight_step(j, s0v[0], nm0, pr, p0[0], l_run[0], masked, thr0); });
        v0h[i] = read_v(i, cv, 0);
        __builtin_amdgcn_sched_barrier(0);
      });
      // C
      zero(s1v[0]);
      static_for<0, KS>([&](auto i) {
        s1v[0] = PElem<DT>::mfma(k1[i], qf[0][i], s1v[0]);
        static_for<i * 9 / KS, (i + 1) * 9 / KS>([&](auto j) { weight_step(j, s0v[1], nm1, pr, p0[1], l_run[1], masked, thr1); });
        v0h[KS + i] = read_v(std::integral_constant<int, KS + i>{}, cv, 0);
        __builtin_amdgcn_sched_barrier(0);
      });
      // D
      zero(s1v[1]);
      static_for<0, KS>([&](auto i) {
        s1v[1] = PElem<DT>::mfma(k1[i], qf[1][i], s1v[1]);
        static_for<i * 9 / KS, (i + 1) * 9 / KS>([&](auto j) { weight_step(j, s1v[0], nm0, pr, p1[0], l_run[0], masked, thr0 - 32); });
        __builtin_amdgcn_sched_barrier(0);
      });
      // E
      static_for<0, NPV>([&](auto i) {
        pv_mfma(i, v0h, p0);
        static_for<i * 9 / NPV, (i + 1) * 9 / NPV>([&](auto j) { weight_step(j, s1v[1], nm1, pr, p1[1], l_run[1], masked, thr1 - 32); });
        v1h[i] = read_v(i, cv, 1);
        __builtin_amdgcn_sched_barrier(0);
      });
      sync_next();
      // F
      static_for<0, NPV>([&](auto i) {
        pv_mfma(i, v1h, p1);
        if constexpr (i < KS) {
          k_at[i] += k_step;
          k0[i] = lds_read16(k_at[i]);
        }
        if constexpr (i == 0 && NLD > 2) issue_part(part3, t2, gk);
        if constexpr (i == NPV / 2) issue_part(part0, t3, fk);
        __builtin_amdgcn_sched_barrier(0);
      });
      t2 = t3;
    } else {
      // Two wavefronts per SIMD, 32 rows each: four stages of eight slots, the same slot discipline.  What one
      // wavefront's slots leave idle (waits for LDS, the barrier) the other wavefront of the SIMD fills, so the
      // operand reads run only two slots ahead of their MFMA (a wavefront has 256 registers here):
      //   A  S(block 0)                    | issues a load of tile kt+2
      //   B  S(block 1)                    | weights of A's scores
      //   C  O += V(block 0) P(block 0)    | weights of B's scores
      //   -- synchronisation point --
      //   D  O += V(block 1) P(block 1)    | issues a load of tile kt+3
      // Operands in the order the 32 slots consume them: K block 0 (8 reads), K block 1 (8), V block 0 (8 pairs of
      // transposing reads), V block 1 (8 pairs), then K block 0 of the next tile: slot n issues the read of slot n+2.
      // k0[0] and k0[1] hold the first two operands on entry and those of the next tile on exit; k_at[j] moves on to
      // the next tile's buffer right after its last use in this one.
      static_assert(RB == 2 || (NLD == 2 && NPV == KS && NVR == 2 * KS), "slot plan of the 32-row tile");
      f32x16 s0v, s1v;
      u32x4 p0[1][2], p1[1][2];
      u32x4 k1[KS];
      u32x2 v0h[NVR], v1h[NVR];
      float pr[16];
      const float nm0 = -m_used[0];
      const char* cv = ck + TILEB;
      const uint32_t k_step = (uint32_t)uni((int)(lds_addr_of(nk) - lds_addr_of(ck)));
      int thr0 = 0;
      if constexpr (decltype(masked)::value) {
        const Tile cur = tile_of(kt);
        thr0 = min(lim[0] - cur.jbase, cur.last_row) - 4 * hi;
      }
      Tile t3;
      if (__builtin_expect(kt + 3 < run_end, 1)) {
        t3.k = t2.k + (size_t)kBN * row_bytes;
        t3.v = t2.v + (size_t)kBN * row_bytes;
        t3.last_row = kBN - 1;
        t3.jbase = 0;
      } else {
        t3 = tile_ahead(kt + 3);
        run_end = run_end_of(kt + 3);
      }
      // the read that slot n of the tile issues (n = 0 .. 31)
      auto ahead = [&](auto nc) {
        constexpr int n = decltype(nc)::value + 2;  // the slot it is for
        if constexpr (n < KS) {
          k0[n] = lds_read16(k_at[n]);
        } else if constexpr (n < 2 * KS) {
          k1[n - KS] = lds_read16(k_at[n - KS] + 32 * ROWB);
          k_at[n - KS] += k_step;
        } else if constexpr (n < 3 * KS) {
          constexpr int m = n - 2 * KS;
          v0h[2 * m] = read_v(std::integral_constant<int, 2 * m>{}, cv, 0);
          v0h[2 * m + 1] = read_v(std::integral_constant<int, 2 * m + 1>{}, cv, 0);
        } else if constexpr (n < 4 * KS) {
          constexpr int m = n - 3 * KS;
          v1h[2 * m] = read_v(std::integral_constant<int, 2 * m>{}, cv, 1);
          v1h[2 * m + 1] = read_v(std::integral_constant<int, 2 * m + 1>{}, cv, 1);
        } else {
          k0[n - 4 * KS] = lds_read16(k_at[n - 4 * KS]);
        }
      };
      // A
      zero(s0v);
      static_for<0, KS>([&](auto i) {
        s0v = PElem<DT>::mfma(k0[i], qf[0][i], s0v);
        ahead(i);
        if constexpr (i == 0) issue_part(part1, t2, gk);
        __builtin_amdgcn_sched_barrier(0);
      });
      // B
      zero(s1v);
      static_for<0, KS>([&](auto i) {
        s1v = PElem<DT>::mfma(k1[i], qf[0][i], s1v);
        static_for<i * 9 / KS, (i + 1) * 9 / KS>([&](auto j) { weight_step(j, s0v, nm0, pr, p0[0], l_run[0], masked, thr0); });
        ahead(std::integral_constant<int, KS + i>{});
        __builtin_amdgcn_sched_barrier(0);
      });
      // C
      static_for<0, NPV>([&](auto i) {
        pv_mfma(i, v0h, p0);
        static_for<i * 9 / NPV, (i + 1) * 9 / NPV>([&](auto j) { weight_step(j, s1v, nm0, pr, p1[0], l_run[0], masked, thr0 - 32); });
        ahead(std::integral_constant<int, 2 * KS + i>{});
        __builtin_amdgcn_sched_barrier(0);
      });
      sync_next();
      // D
      static_for<0, NPV>([&](auto i) {
        pv_mfma(i, v1h, p1);
        ahead(std::integral_constant<int, 3 * KS + i>{});
        if constexpr (i == NPV / 2) issue_part(part0, t3, fk);
        __builtin_amdgcn_sched_barrier(0);
      });
      t2 = t3;
    }
  };

  auto buf_of = [&](int i) -> char* { return lds_tiles + (i & 3) * (2 * TILEB); };

  // Generic tile: masked (ragged end of a segment, causal diagonal), classic online softmax (reference maxima
  // follow the data, accumulators rescaled when a maximum moves by more than kTau).  Row r of the tile is
  // visible to a query row iff it exists and its position jbase + r does not exceed the row's limit.
  auto generic_tile = [&](const char* tk, const Tile& tl) {
    const char* tv = tk + TILEB;
    int vis[RB];
#pragma unroll
    for (int cb = 0; cb < RB; ++cb) vis[cb] = min(lim[cb] - tl.jbase, tl.last_row);
#pragma unroll 1
    for (int kb = 0; kb < 2; ++kb) {
      f32x16 s[RB];
      scores(tk, kb, s);
#pragma unroll
      for (int cb = 0; cb < RB; ++cb)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int r = 32 * kb + 8 * (i >> 2) + 4 * hi + (i & 3);
          s[cb][i] = r <= vis[cb] ? s[cb][i] : -INFINITY;
        }
      float tmax[RB];
      block_max(s, tmax);
      bool grows[RB], any_grow = false;
#pragma unroll
      for (int cb = 0; cb < RB; ++cb) {
        grows[cb] = tmax[cb] > m_used[cb] + kTau;
        any_grow |= grows[cb];
      }
      if (__builtin_amdgcn_ballot_w64(any_grow) != 0) {
        // The accumulators live in accumulation registers (the MFMAs read and write them there); this is the
        // only other code that touches them, so it goes through explicit moves.
#pragma unroll
        for (int cb = 0; cb < RB; ++cb) {
          const bool grow = grows[cb];
          const float m_new = grow ? tmax[cb] : m_used[cb];
          // (a row that does not move may still be without a maximum: -inf - -inf must not reach the exponential)
          const float alpha = grow ? __builtin_amdgcn_exp2f(m_used[cb] - m_new) : 1.0f;
          m_used[cb] = m_new;
          l_run[cb] *= alpha;
#pragma unroll
          for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              if constexpr (RB == 2) {
                float t;
                asm volatile("v_accvgpr_read_b32 %1, %0\n\tv_mul_f32 %1, %1, %2\n\ts_nop 0\n\tv_accvgpr_write_b32 %0, %1"
                             : "+a"(acc[db][cb][i]), "=&v"(t)
                             : "v"(alpha));
              } else {
                acc[db][cb][i] *= alpha;
              }
            }
        }
      }
      u32x4 pf[RB][2];
      weights(s, pf);
      u32x2 vh[NVR];
      static_for<0, NVR>([&](auto r) { vh[r] = read_v(r, tv, kb); });
      static_for<0, NPV>([&](auto i) { pv_mfma(i, vh, pf); });
    }
  };

  // Workgroup barrier for data exchanged through LDS: waits for this wavefront's LDS operations only (the barrier
  // of __syncthreads would wait for the tile loads in flight as well).
  auto lds_barrier = []() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

  // acc[db][cb][i] is d = 32*db + 8*(i/4) + 4*hi + i%4 of the lane's query row (cb*32 + col of the wavefront's 64).
  // out[row, d] = acc * inv.  The rows go through LDS, 32 values of each at a time, so that the global stores are
  // whole 16-byte pieces of 64 contiguous bytes per row rather than 8 bytes per lane scattered over 32 rows.
  auto write_rows = [&](const Piece& pc, const float* inv) {
    const int tok0 = pc.t * tb, nt = min(tb, pc.N - tok0);
    char* stg = lds_stage[wave];
    const unsigned g_magic = (65536u + (unsigned)G - 1u) / (unsigned)G;  // r / G for r < 256
#pragma unroll
    for (int db = 0; db < DB; ++db) {
#pragma unroll
      for (int cb = 0; cb < RB; ++cb) {
        char* sp = stg + (cb * 32 + col) * STG + 8 * hi;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          u32x2 w;
          w[0] = PElem<DT>::pack2(acc[db][cb][4 * q4] * inv[cb], acc[db][cb][4 * q4 + 1] * inv[cb]);
          w[1] = PElem<DT>::pack2(acc[db][cb][4 * q4 + 2] * inv[cb], acc[db][cb][4 * q4 + 3] * inv[cb]);
          *(u32x2*)(sp + 16 * q4) = w;
        }
      }
      // (LDS operations of one wavefront complete in order: no barrier between the writes above and these reads,
      // nor between these reads and the next round's writes)
#pragma unroll
      for (int i = 0; i < 2 * RB; ++i) {
        const int rl = 16 * i + lane / 4, ch = lane % 4;
        const int rr = wave * WR + rl;
        const int t = (int)(((unsigned)rr * g_magic) >> 16), head = rr - t * G;
        const u32x4 v = *(const u32x4*)(stg + rl * STG + ch * 16);
        if (t < nt)
          *(u32x4*)(p.out + ((size_t)(pc.cu_b + tok0 + t) * p.hq + (size_t)pc.g * G + head) * ROWB + db * 64 +
                    ch * 16) = v;
      }
    }
  };

  // Piece slots in the workspace.  A slot holds, for the 256 rows, the reference maxima, the sums and the
  // unnormalised accumulators of one piece in the order the lanes hold them: thread t's accumulator values
  // (db, cb, 4 consecutive i) are the 16 bytes at block ((db*RB + cb)*4 + i/4), position t - every store and load of
  // the workgroup covers 4 or 8 KiB contiguous.  Rows are the same in every workgroup (row = 32*RB*wave + 32*cb + col).
  auto slot_of = [&](uint32_t owner, bool head) -> float* {
    return p.ws + (size_t)(2 * owner + (head ? 1u : 0u)) * piece_floats(D);
  };

  int gt = 0;           // position of the current tile in the stream; its buffer is gt % 4
  bool primed = false;  // the first tiles of the piece are already on their way (issued by the previous piece)
  for (;;) {
    // ---- the piece: tiles s0 .. s1-1 of item (b, g, t) ----
    s0 = cur.s0;
    s1 = cur.s1;
    P = cur.P;
    const int tok0 = cur.t * tb;
    ntok = min(tb, cur.N - tok0);
    const int nfast_item = cur.fastA + cur.fastB;
#pragma unroll
    for (int cb = 0; cb < RB; ++cb) {
      const int t = (wave * WR + cb * 32 + col) / G;
      lim[cb] = P + tok0 + min(t, ntok - 1);  // key j is visible iff j <= lim
    }
    // Rows past the last token of the tile are padding; a wavefront whose 64 rows are all padding computes nothing.
    wave_idle = (wave * WR) / G >= ntok;
    // The tiles after this piece are first asked for by its third-last tile; in a piece of four tiles or more the
    // look-up runs beside the second tile (scalar work next to the matrix pipe) instead of in front of the first.
    int park_at = s1 - s0 >= 4 ? s0 + 1 : s0 - 1;
    if (park_at < s0) park_ahead();

    // Fast tiles of this piece: s0 .. nf-1.
    int nf = min(s1, nfast_item);
    Piece nxt;
    u32x4 qn[RB][KS];
    for (int attempt = 0;; ++attempt) {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int cb = 0; cb < RB; ++cb) zero(acc[db][cb]);
#pragma unroll
      for (int cb = 0; cb < RB; ++cb) {
        m_used[cb] = -INFINITY;
        l_run[cb] = 0.f;
      }

      Tile t2;
      run_end = run_end_of(s0 + 2);
      if (!primed) {
        issue_tile(tile_ahead(s0), buf_of(gt));
        issue_tile(tile_ahead(s0 + 1), buf_of(gt + 1));
        t2 = tile_ahead(s0 + 2);
        issue_part(part0, t2, buf_of(gt + 2));
        wait_loads(std::integral_constant<int, VM + 2>{});
        __builtin_amdgcn_s_barrier();
        primed = true;
      } else {
        // (the last tile of the previous piece left tile s0 landed, s0+1 issued and the first load of s0+2 issued)
        t2 = tile_ahead(s0 + 2);
      }
      // The Q operands stay in accumulation registers (MFMA reads its B operand from there as well), which leaves
      // the vector registers to the scores, the weights and the in-flight LDS operand reads.  They are pinned
      // there only now, so that their loads and the first tiles' loads are in flight together.
      if constexpr (RB == 2) {
#pragma unroll
        for (int cb = 0; cb < RB; ++cb)
#pragma unroll
          for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+a"(qf[cb][ks]));
      }
      int kt = s0;
      if (wave_idle) {
        // No row of this wavefront belongs to a token (the last token tile of a request is padded to 256 rows): it
        // only keeps its part of the tile pipeline going - the same loads, waits and barriers per tile as below.
        for (; kt < s1; ++kt, ++gt) {
          if (kt == park_at) park_ahead();
          issue_before_sync(t2, buf_of(gt + 2));
          sync_next();
          const Tile t3 = tile_ahead(kt + 3);
          issue_after_sync(t2, t3, buf_of(gt + 2), buf_of(gt + 3));
          t2 = t3;
        }
      } else if (kt < nf) {
        // Reference maxima for the fast tiles: the column maxima of the first 32 keys.  fp16 weights have a short
        // exponent range (2^-24 .. 2^16), and only an overflow is noticed afterwards (rows whose later scores
        // outgrow the representable range are caught below), never an underflow: the reference sits 8 units BELOW
        // the maxima, so that a key as good as the first ones weighs 2^8, later keys may exceed them by 2^8 more
        // before the fallback is taken, and keys 2^22 times lighter than the first ones still keep every bit.
        u32x4 k0[KS];
        {
          const char* first = buf_of(gt);
          static_for<0, KS>([&](auto ks) {
            k_at[ks] = lds_addr_of(first + col * ROWB + (((2 * ks + hi) ^ kswz) * 16));
            k0[ks] = lds_read16(k_at[ks]);
          });
          f32x16 s[RB];
          float tmax[RB];
#pragma unroll
          for (int cb = 0; cb < RB; ++cb) zero(s[cb]);
          static_for<0, KS>([&](auto ks) {
#pragma unroll
            for (int cb = 0; cb < RB; ++cb) s[cb] = PElem<DT>::mfma(k0[ks], qf[cb][ks], s[cb]);
          });
          block_max(s, tmax);
#pragma unroll
          for (int cb = 0; cb < RB; ++cb) m_used[cb] = tmax[cb] - (DT == VT_F16 ? 8.0f : 0.0f);
        }
        for (; kt < nf; ++kt, ++gt) {
          if (kt == park_at) park_ahead();
          fast_tile(std::false_type{}, kt, buf_of(gt), buf_of(gt + 1), buf_of(gt + 2), buf_of(gt + 3), k0, t2);
        }
        // The masked tiles that follow fast ones keep the fixed reference maxima (every row has one by now) and
        // the same instruction schedule, with the mask applied to the weights.
        for (; kt < s1; ++kt, ++gt) {
          if (kt == park_at) park_ahead();
          fast_tile(std::true_type{}, kt, buf_of(gt), buf_of(gt + 1), buf_of(gt + 2), buf_of(gt + 3), k0, t2);
        }
      }
      for (; kt < s1; ++kt, ++gt) {
        if (kt == park_at) park_ahead();
        issue_before_sync(t2, buf_of(gt + 2));
        generic_tile(buf_of(gt), tile_of(kt));
        sync_next();
        const Tile t3 = tile_ahead(kt + 3);
        issue_after_sync(t2, t3, buf_of(gt + 2), buf_of(gt + 3));
        t2 = t3;
      }
      // The next piece, and its query rows on their way while this piece's results go out.
      if (attempt == 0) {
        nxt = next_piece(cur);
        if (nxt.valid) load_q(nxt, qn);
      }
      if (attempt > 0 || nf <= s0) break;
      // Fixed reference maxima can overflow the weights when later scores are far larger than the first ones: then
      // some sum or accumulator is no longer finite and the whole workgroup redoes the piece the classic way.
      float chk = 0.f;
#pragma unroll
      for (int cb = 0; cb < RB; ++cb) {
        chk += l_run[cb];
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i) chk += __builtin_fabsf(acc[db][cb][i]);
      }
      const bool bad = __builtin_amdgcn_ballot_w64(!(chk < INFINITY)) != 0;
      if (lane == 0) s_vote[wave] = bad ? 1 : 0;
      lds_barrier();
      int votes = 0;
#pragma unroll
      for (int w = 0; w < NW; ++w) votes |= s_vote[w];
      const int any_bad = uni(votes);
      lds_barrier();  // (nobody writes the votes of the next piece before everybody has read these)
      if (!any_bad) break;
      // Start over from the piece's first tile: nothing may be in flight into the buffers, nobody may still read them.
      wait_loads(std::integral_constant<int, 0>{});
      __builtin_amdgcn_s_barrier();
      primed = false;
      nf = s0;
    }

    float l_tot[RB];
#pragma unroll
    for (int cb = 0; cb < RB; ++cb) l_tot[cb] = l_run[cb] + __shfl_xor(l_run[cb], 32);
    bool finish = s0 == 0 && s1 == cur.nkt;  // the piece is the whole item
    if (!finish) {
      // The item is shared with other workgroups.  Its pieces meet in the workspace: whoever finishes a piece adds
      // one to the item's arrival count; the one who finds all the others already there merges their slots into its
      // own registers and writes the output, everybody else leaves the piece in its slot.  Nobody waits for anybody.
      // The count lives in the word of the group that owns the item's first tile, tagged with the number of this
      // launch (a count left by an earlier launch reads as zero).
      const uint32_t n = p.n_groups, total = p.total_cost;
      const uint32_t unit0 = cur.item_begin + (uint32_t)kItemCost;  // first cost unit of the item's first tile
      uint32_t w0 = (uint32_t)((((uint64_t)unit0 + 1) * n - 1) / total);
      while (group_begin(total, n, w0 + 1) <= unit0) ++w0;
      while (group_begin(total, n, w0) > unit0) --w0;
      ItemShape sh;
      sh.nkt = cur.nkt;
      sh.nfast = cur.nfast;
      const uint32_t cost = item_cost(sh);
      // groups w0 .. w_last hold tiles of the item; `others` of them apart from this one
      uint32_t w_last = w0, pieces = 0;
      for (uint32_t u = w0;; ++u) {
        const uint32_t c0 = u == w0 ? 0u : group_begin(total, n, u) - cur.item_begin;
        const uint32_t c1 = min(cost, group_begin(total, n, u + 1) - cur.item_begin);
        if (tile_at(sh, c1) > tile_at(sh, c0)) {
          ++pieces;
          w_last = u;
        }
        if (c1 >= cost) break;
      }
      unsigned long long* word = p.arrivals + w0;
      const unsigned long long tag = p.launch << 16;
      auto count_of = [&](unsigned long long v) -> uint32_t { return (v >> 16) == p.launch ? (uint32_t)(v & 0xffffu) : 0u; };
      if (tid == 0)
        s_arrived = count_of(__hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
      lds_barrier();
      bool last = (uint32_t)uni((int)s_arrived) == pieces - 1;
      lds_barrier();
      if (!last) {
        // leave the piece in the slot (stores that go through to memory), wait until they have landed, then count it
        float* sl = slot_of(group, group == w0);
        if (!wave_idle) {
#pragma unroll
          for (int cb = 0; cb < RB; ++cb) {
            if (hi == 0) {
              __hip_atomic_store(sl + wave * WR + cb * 32 + col, m_used[cb], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              __hip_atomic_store(sl + 256 + wave * WR + cb * 32 + col, l_tot[cb], __ATOMIC_RELAXED,
                                 __HIP_MEMORY_SCOPE_AGENT);
            }
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
              for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 w = {acc[db][cb][4 * q4], acc[db][cb][4 * q4 + 1], acc[db][cb][4 * q4 + 2],
                                 acc[db][cb][4 * q4 + 3]};
                store16_device(sl + 512 + (size_t)(((db * RB + cb) * 4 + q4) * NT + tid) * 4, w);
              }
          }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        lds_barrier();
        if (tid == 0) {
          unsigned long long seen = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          uint32_t before;
          do {
            before = count_of(seen);
          } while (!__hip_atomic_compare_exchange_strong(word, &seen, tag | (before + 1), __ATOMIC_RELAXED,
                                                         __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
          s_arrived = before;
        }
        lds_barrier();
        last = (uint32_t)uni((int)s_arrived) == pieces - 1;
        lds_barrier();
      }
      if (last) {
        if (!wave_idle) {
          for (uint32_t u = w0; u <= w_last; ++u) {
            if (u == group) continue;
            const uint32_t c0 = u == w0 ? 0u : group_begin(total, n, u) - cur.item_begin;
            const uint32_t c1 = min(cost, group_begin(total, n, u + 1) - cur.item_begin);
            if (tile_at(sh, c1) <= tile_at(sh, c0)) continue;
            const float* sl = slot_of(u, u == w0);
#pragma unroll
            for (int cb = 0; cb < RB; ++cb) {
              const int r = wave * WR + cb * 32 + col;
              f32x4 o[4 * DB];
#pragma unroll
              for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
                  load16_device(o[4 * db + q4], sl + 512 + (size_t)(((db * RB + cb) * 4 + q4) * NT + tid) * 4);
              const float m_o = __hip_atomic_load(sl + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              const float l_o = __hip_atomic_load(sl + 256 + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              static_assert(DB == 4 || DB == 2, "operand list below");
              if constexpr (DB == 4)
                asm volatile("s_waitcnt vmcnt(0)"
                             : "+v"(o[0]), "+v"(o[1]), "+v"(o[2]), "+v"(o[3]), "+v"(o[4]), "+v"(o[5]), "+v"(o[6]),
                               "+v"(o[7]), "+v"(o[8]), "+v"(o[9]), "+v"(o[10]), "+v"(o[11]), "+v"(o[12]), "+v"(o[13]),
                               "+v"(o[14]), "+v"(o[15])
                             :
                             : "memory");
              else
                asm volatile("s_waitcnt vmcnt(0)"
                             : "+v"(o[0]), "+v"(o[1]), "+v"(o[2]), "+v"(o[3]), "+v"(o[4]), "+v"(o[5]), "+v"(o[6]),
                               "+v"(o[7])
                             :
                             : "memory");
              const float m_new = fmaxf(m_used[cb], m_o);
              // (a side that has seen no key has no maximum: weight 0, and never the exponential of inf - inf)
              const float a = m_used[cb] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_used[cb] - m_new);
              const float bwt = m_o == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_o - m_new);
              m_used[cb] = m_new;
              l_tot[cb] = l_tot[cb] * a + l_o * bwt;
#pragma unroll
              for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4)
#pragma unroll
                  for (int i = 0; i < 4; ++i)
                    acc[db][cb][4 * q4 + i] = acc[db][cb][4 * q4 + i] * a + o[4 * db + q4][i] * bwt;
            }
          }
        }
        finish = true;
      }
    }
    if (finish) {
      float inv[RB];
#pragma unroll
      for (int cb = 0; cb < RB; ++cb) inv[cb] = 1.0f / l_tot[cb];
      write_rows(cur, inv);
    }
    if (!nxt.valid) break;
    cur = nxt;
#pragma unroll
    for (int cb = 0; cb < RB; ++cb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) qf[cb][ks] = qn[cb][ks];
  }  // piece loop
  // nothing may still be on its way into LDS when the workgroup ends
  wait_loads(std::integral_constant<int, 0>{});
}

}  // namespace

// Host mirror of the kernel's decomposition: same helpers, same order.
int plan_prefill(const vt_ctx* ctx, const int32_t* cu_host, const int32_t* plens_host, uint32_t batch, uint32_t hq,
                 uint32_t hkv, uint32_t d, bool split, vt_prefill_plan* out, vt_prefill_piece* pieces,
                 uint64_t max_pieces, uint64_t* n_pieces) {
  if (!cu_host || !plens_host || !out || !hq || !hkv || hq % hkv) return VT_E_INVALID;
  const uint32_t G = hq / hkv;
  if (G > (uint32_t)kRows || batch > (uint32_t)kMaxPrefillBatch || (d != 64 && d != 128)) return VT_E_UNSUPPORTED;
  if ((uint64_t)hkv * d * 2 >= (1u << 24)) return VT_E_UNSUPPORTED;  // 24-bit row offsets in the tile loads
  const int tb = kRows / (int)G;
  uint64_t total = 0, tiles = 0, items = 0;
  for (uint32_t b = 0; b < batch; ++b) {
    const int n = cu_host[b + 1] - cu_host[b], P = plens_host[b];
    if (n < 0 || P < 0) return VT_E_INVALID;
    if ((int64_t)P + n > 0x3fffffff) return VT_E_UNSUPPORTED;
    total += (uint64_t)request_cost(P, n, tb, split) * hkv;
    for (int t = 0; t * tb < n; ++t) tiles += (uint64_t)item_shape(P, n, t, tb, split).nkt * hkv;
    items += (uint64_t)((n + tb - 1) / tb) * hkv;
    if (total > 0x7fffffffull) return VT_E_UNSUPPORTED;
  }
  uint64_t groups = total / kMinCostPerGroup;
  groups = groups < 1 ? 1 : (groups > (uint64_t)ctx->n_cus ? (uint64_t)ctx->n_cus : groups);
  out->total_cost = total;
  out->n_tiles = tiles;
  out->n_items = (uint32_t)items;
  out->n_groups = total ? (uint32_t)groups : 0;
  out->workspace_bytes = total ? 2 * groups * piece_floats((int)d) * sizeof(float) : 0;
  uint64_t count = 0;
  if ((pieces || n_pieces) && total) {
    // walk the items once, carving each at the group boundaries that fall inside it
    uint64_t begin = 0;  // first cost unit of the current item
    for (uint32_t b = 0; b < batch; ++b) {
      const int n = cu_host[b + 1] - cu_host[b], P = plens_host[b];
      for (uint32_t g = 0; g < hkv; ++g)
        for (int t = 0; t * tb < n; ++t) {
          const ItemShape sh = item_shape(P, n, t, tb, split);
          const uint64_t cost = item_cost(sh);
          // groups whose range intersects [begin, begin + cost)
          uint32_t w = (uint32_t)(begin * groups / total);  // its range starts at or before `begin`
          while (group_begin((uint32_t)total, (uint32_t)groups, w + 1) <= begin) ++w;
          for (; w < groups && group_begin((uint32_t)total, (uint32_t)groups, w) < begin + cost; ++w) {
            const uint64_t lo = group_begin((uint32_t)total, (uint32_t)groups, w);
            const uint64_t hi = group_begin((uint32_t)total, (uint32_t)groups, w + 1);
            const uint32_t c0 = (uint32_t)(lo > begin ? lo - begin : 0);
            const uint32_t c1 = (uint32_t)(hi < begin + cost ? hi - begin : cost);
            const int s0 = tile_at(sh, c0), s1 = tile_at(sh, c1);
            if (s1 <= s0) continue;
            if (pieces && count < max_pieces) {
              vt_prefill_piece& pc = pieces[count];
              pc.group = w;
              pc.request = b;
              pc.kv_head = g;
              pc.token_tile = (uint32_t)t;
              pc.tile_begin = (uint32_t)s0;
              pc.tile_end = (uint32_t)s1;
              pc.n_tiles = (uint32_t)sh.nkt;
              pc.n_fast = (uint32_t)sh.nfast;
            }
            ++count;
          }
          begin += cost;
        }
    }
  }
  if (n_pieces) *n_pieces = count;
  return VT_OK;
}

int launch_prefill(vt_ctx* ctx, const vt_prefill_args* a, void* stream) {
  const uint32_t G = a->n_q_heads / a->n_kv_heads;
  const bool split = a->k_new != nullptr;
  vt_prefill_plan plan;
  int rc = plan_prefill(ctx, a->cu_seqlens_host, a->prefix_lens_host, a->batch, a->n_q_heads, a->n_kv_heads,
                        a->head_dim, split, &plan, nullptr, 0, nullptr);
  if (rc != VT_OK) return rc;
  if (plan.total_cost == 0) return VT_OK;
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
  // A zero scale (every visible key weighs the same) runs as the smallest positive one: the scaled scores then vanish
  // in fp32 and masked keys (minus infinity before scaling) stay masked.
  p.scale_log2e = std::fmax(std::fabs(a->scale) * 1.4426950408889634f, 1.17549435e-38f);
  p.q_sign = a->scale < 0.0f ? 0x80008000u : 0u;
  p.total_cost = (uint32_t)plan.total_cost;
  p.n_groups = plan.n_groups;
  rc = ensure_workspace(ctx, plan.workspace_bytes);
  if (rc != VT_OK) return rc;
  if (!ctx->arrivals || plan.n_groups > kMaxPrefillGroups) return VT_E_UNSUPPORTED;
  p.ws = (float*)ctx->ws;
  p.arrivals = (unsigned long long*)ctx->arrivals;
  p.launch = ++ctx->prefill_launches;
  hipStream_t st = (hipStream_t)stream;
  // head_dim 128: eight wavefronts of 32 rows (two per SIMD); head_dim 64: four wavefronts of 64 rows.
  const bool narrow = a->head_dim == 128 && !ctx->prefill_wide;
  const dim3 grid(p.n_groups), block(narrow ? 512 : 256);
  prof_begin(ctx, 1, st);
  if (a->dtype == VT_BF16 && a->head_dim == 128) {
    if (narrow)
      hipLaunchKernelGGL((prefill_kernel<VT_BF16, 128, 1>), grid, block, 0, st, p);
    else
      hipLaunchKernelGGL((prefill_kernel<VT_BF16, 128, 2>), grid, block, 0, st, p);
  } else if (a->dtype == VT_BF16 && a->head_dim == 64) {
    hipLaunchKernelGGL((prefill_kernel<VT_BF16, 64, 2>), grid, block, 0, st, p);
  } else if (a->dtype == VT_F16 && a->head_dim == 128) {
    if (narrow)
      hipLaunchKernelGGL((prefill_kernel<VT_F16, 128, 1>), grid, block, 0, st, p);
    else
      hipLaunchKernelGGL((prefill_kernel<VT_F16, 128, 2>), grid, block, 0, st, p);
  } else {
    hipLaunchKernelGGL((prefill_kernel<VT_F16, 64, 2>), grid, block, 0, st, p);
  }
  prof_end(ctx, st);
  return hipGetLastError() == hipSuccess ? VT_OK : VT_E_DRIVER;
}

}  // namespace vt
