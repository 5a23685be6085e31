// The expert networks over the loaded experts (Eq. (2)/(7)/(8)) and the weighted combine.
//
// E_i(x) = W_down,i ( silu(W_gate,i x) * (W_up,i x) ) is evaluated per segment (one expert, the
// hidden rows of its (token, slot) pairs) in two passes over that expert's weights:
//   pass 1  act[p, :] = silu(W_gate x_p) * (W_up x_p)        streams W_gate,i and W_up,i once
//   pass 2  y[pair, :] = W_down act[p, :]                    streams W_down,i once
// and a final combine adds the k weighted rows of every token in slot order (deterministic).
//
// bf16 path.  Weight rows are the MFMA "A" side (v_mfma_f32_16x16x32_bf16), tokens the "B" side
// (16 per tile, up to 8 tiles per pass, so a segment of up to 128 pairs reads its expert once).
// Work is cut into equal-byte items: a workgroup of 4 waves takes 128 weight rows (32 per wave)
// of one expert and walks K in chunks; however uneven the segment sizes, every compute unit
// streams the same number of weight bytes.  Per chunk each wave loads its rows with fully
// coalesced 16-byte loads, parks them in a wave-private, XOR-swizzled LDS tile and reads them
// back in MFMA operand layout; the token chunk is loaded once per workgroup into a shared LDS
// tile (double-buffered up to 4 token tiles; one 32 KB buffer and a second barrier for 8).  (Loading
// operands from global memory directly in MFMA layout costs a cache-line lookup per lane and saturates
// the texture-address path long before HBM.)  A segment of more than 128 pairs is cut into pieces that
// are work items of their own: its walks over the expert run side by side, not one after the other.
// Workgroups start their K walk at staggered offsets: weight rows are a power-of-two stride
// apart, and equal offsets would pile the concurrent reads onto the same memory channels.
// Shapes whose K is not a multiple of 128 take a simpler direct-load variant of the same tiling.
// The intermediate act and the per-pair outputs y are indexed by the flat pair id t * k + slot.
//
// Where its segment comes from: either from the segment arrays (seg_expert, seg_off, perm; any
// caller), or - inside the fused layer, for small trees - every workgroup derives it from the
// shortlist, the pair count of every shortlisted expert and the restricted routing table, which takes
// no longer than reading perm and spares the budget stage its serial grouping step.
#include "common.h"

namespace moespec {

constexpr int kFfnThreads = 256;
static_assert(kSelfMaxExperts <= kFfnThreads, "one thread per shortlist rank");
constexpr int kFfnWaves = kFfnThreads / kWave;
constexpr int kMaxTiles = 8;  // token tiles of 16 per pass over the weights

// A segment is processed only if it names a real expert and lies inside the pair table; pair
// indices are clamped into [0, M*k) so that malformed tables cannot address outside the buffers.
__device__ __forceinline__ bool segment_ok(int e, int beg, int m, long long list_len, int N) {
  return e >= 0 && e < N && m > 0 && beg >= 0 && (long long)beg + m <= list_len;
}
__device__ __forceinline__ int pair_index(const int32_t *perm, int pos, int M, int k) {
  const int q = perm[pos];
  return q < 0 ? 0 : (q >= M * k ? M * k - 1 : q);
}

// base + a 32-bit byte offset: with a uniform base the load needs one offset register, not a 64-bit address
__device__ __forceinline__ const uint16_t *at_bytes(const uint16_t *base, uint32_t bytes) {
  return reinterpret_cast<const uint16_t *>(reinterpret_cast<const char *>(base) + bytes);
}
__device__ __forceinline__ bf16x8 ld_frag(const uint16_t *p) { return *reinterpret_cast<const bf16x8 *>(p); }
// Weight bytes are read exactly once: load them with the non-temporal hint so that the stream does
// not push the (re-read) token rows out of the caches.
__device__ __forceinline__ bf16x8 ld_stream(const uint16_t *p) {
  return __builtin_nontemporal_load(reinterpret_cast<const bf16x8 *>(p));
}

// acc0[j] += A0 . B_j, acc1[j] += A1 . B_j over K, for NT token tiles; U K-steps of 32 per stage,
// two register stages so that the next stage's loads are in flight during the current MFMAs.
// a0/a1/bp[] are per-lane pointers (already offset by the lane's row and K group).  K % (32 U) == 0.
// The walk over K starts at element ks (a multiple of 32 U) and wraps: waves that start at
// different offsets spread the concurrent row reads over the memory channels (rows of a weight
// matrix are a power-of-two stride apart, so equal offsets would pile onto the same channels).
template <int NT, int U>
__device__ __forceinline__ void stream_rows(const uint16_t *a0, const uint16_t *a1, const uint16_t *const (&bp)[NT],
                                            int K, int ks, f32x4 (&acc0)[NT], f32x4 (&acc1)[NT]) {
  bf16x8 A0[2][U], A1[2][U], Bf[2][U][NT];
  auto load = [&](int st, int k0) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      A0[st][u] = ld_frag(a0 + k0 + 32 * u);
      A1[st][u] = ld_frag(a1 + k0 + 32 * u);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int j = 0; j < NT; ++j) Bf[st][u][j] = ld_frag(bp[j] + k0 + 32 * u);
  };
  auto compute = [&](int st) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        acc0[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A0[st][u], Bf[st][u][j], acc0[j], 0, 0, 0);
        acc1[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A1[st][u], Bf[st][u][j], acc1[j], 0, 0, 0);
      }
  };
  constexpr int KS = 32 * U;
  const int nst = K / KS;
  int k = (ks / KS) * KS;
  load(0, k);
  for (int i = 0; i < nst; i += 2) {
    int k1 = k + KS;
    k1 = k1 >= K ? k1 - K : k1;
    if (i + 1 < nst) load(1, k1);
    compute(0);
    k = k1 + KS;
    k = k >= K ? k - K : k;
    if (i + 2 < nst) load(0, k);
    if (i + 1 < nst) compute(1);
  }
}

// Workgroup -> (segment, row tile) for the LDS-tiled passes.  Workgroups are handed to the 8 XCDs
// round-robin by linear id, and each XCD has an L2 of its own and a share of the chip's streaming
// bandwidth.  The work items are the non-empty segments, largest first (a segment of more than 128 pairs
// counts as several, one per piece; "segment" below means work item).  Whole rounds of 8 segments are dealt
// one segment per XCD (all row tiles of a segment get ids that are equal modulo 8, so that its token
// rows are fetched into one L2); the L mod 8 segments left over (all of them when L < 8) have their
// row tiles cut into 8 equal contiguous ranges, one per XCD, so that every XCD streams the same
// number of bytes.  Measured on an idle chip, an XCD places its workgroups on its 32 compute units
// round-robin in id order, two per unit, and a workgroup with many token tiles runs slower than one
// with few (more LDS and matrix work per weight byte); in this order the heavy workgroups of the
// first rounds share their compute unit with the light ones of the later rounds, or with nothing.
// Returns false if the workgroup has no work.  L = number of work items.
constexpr int kXcds = 8;
__device__ __forceinline__ bool xcd_map(int tiles, int L, int &rank, int &tile) {
  const int x = blockIdx.x % kXcds, j = blockIdx.x / kXcds;
  const int full = L / kXcds, rest = L % kXcds;
  if (j < full * tiles) {
    rank = x + kXcds * (j / tiles);
    tile = j % tiles;
    return true;
  }
  const int wr = rest * tiles, lo = wr * x / kXcds, hi = wr * (x + 1) / kXcds;
  const int w = lo + (j - full * tiles);
  rank = full * kXcds + w / tiles;
  tile = w % tiles;
  return w < hi;
}
// items[0].x = number of work items L; items[1 + r] = (segment index, expert, offset, size) of item r: the
// non-empty segments, largest first, each cut into piece_count(size) pieces.  The table has cap + 1 entries.
__device__ __forceinline__ int4 xcd_item(int tiles, int cap, const int4 *__restrict__ items, int &tile, int &rank) {
  int L = items[0].x;
  L = L < 0 ? 0 : (L > cap ? cap : L);
  return xcd_map(tiles, L, rank, tile) ? items[1 + rank] : int4{-1, -1, 0, 0};
}
// The table above built from segment arrays that did not come from the budget stage.  One workgroup.
// Only well-formed segments take part (inside the pair table, at most one pair per token), and only as
// long as their pieces fit the table (they always do when the segments are disjoint).
__global__ __launch_bounds__(256) void segment_items_kernel(const int32_t *__restrict__ seg_expert,
                                                            const int32_t *__restrict__ seg_off, int n_seg, int M,
                                                            int k, int cap, int4 *__restrict__ items) {
  __shared__ int n_items;
  if (threadIdx.x == 0) n_items = 0;
  __syncthreads();
  auto size_of = [&](int j) {
    const int lo = seg_off[j], c = seg_off[j + 1] - lo;
    return (lo >= 0 && c > 0 && c <= M && (long long)lo + c <= (long long)M * k) ? c : 0;
  };
  for (int i = threadIdx.x; i < n_seg; i += blockDim.x) {
    const int c = size_of(i);
    if (c > 0) {
      int first = 0;  // pieces of the segments that rank before this one
      for (int j = 0; j < n_seg; ++j) {
        const int cj = size_of(j);
        first += (cj > c || (cj == c && j < i)) ? piece_count(cj) : 0;
      }
      const int q = piece_count(c), len = (c + q - 1) / q, lo = seg_off[i];
      if (first + q <= cap) {
        for (int p = 0; p < q; ++p)
          items[1 + first + p] = int4{i, seg_expert[i], lo + p * len, min(len, c - p * len)};
        atomicAdd(&n_items, q);
      }
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) items[0] = int4{n_items, 0, 0, 0};
}
// Workgroups of a pass: room for whole rounds of 8 work items.
inline int xcd_grid(int tiles, int n_items) { return kXcds * tiles * ((n_items + kXcds - 1) / kXcds); }

// Start offset (elements) of a wave's walk over K: 128 elements (256 bytes) apart for consecutive waves.
__device__ __forceinline__ int k_stagger(int wave_id, int K) { return (int)(((long long)wave_id * 128) % K); }

__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

// ---- pass 1 (bf16): gate/up projections + SwiGLU ---------------------------------------------
template <int NT, int U>
__device__ __forceinline__ void gateup_tiles(const uint16_t *a0, const uint16_t *a1, const uint16_t *__restrict__ h,
                                             const int32_t *__restrict__ perm, int M, int k, int d, int F, int beg,
                                             int c0, int m, int f0, int ks, uint16_t *__restrict__ act) {
  const int lane = threadIdx.x & 63, col = lane & 15, kg = lane >> 4;
  const uint16_t *bp[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    int p = c0 + j * 16 + col;
    p = p < m ? p : m - 1;  // pad columns repeat the last token; their results are never stored
    const int tok = pair_index(perm, beg + p, M, k) / k;
    bp[j] = h + (size_t)tok * d + kg * 8;
  }
  f32x4 accg[NT], accu[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) accg[j] = accu[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  stream_rows<NT, U>(a0, a1, bp, d, ks, accg, accu);
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int p = c0 + j * 16 + col;
    if (p < m) {
      uint16_t o[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = float_to_bf16_bits(silu_f(accg[j][i]) * accu[j][i]);
      uint2 pk;
      pk.x = (uint32_t)o[0] | ((uint32_t)o[1] << 16);
      pk.y = (uint32_t)o[2] | ((uint32_t)o[3] << 16);
      *reinterpret_cast<uint2 *>(act + (size_t)pair_index(perm, beg + p, M, k) * F + f0 + 4 * kg) = pk;
    }
  }
}

template <int U>
__global__ __launch_bounds__(kFfnThreads, 2) void ffn_gateup_bf16_kernel(
    const uint16_t *__restrict__ h, const uint16_t *__restrict__ w_gate, const uint16_t *__restrict__ w_up,
    const int32_t *__restrict__ seg_expert, const int32_t *__restrict__ seg_off, const int32_t *__restrict__ perm,
    int M, int N, int k, int d, int F, uint16_t *__restrict__ act) {
  const int seg = blockIdx.y;
  const int e = seg_expert[seg];
  const int beg = seg_off[seg], m = seg_off[seg + 1] - beg;
  if (!segment_ok(e, beg, m, (long long)M * k, N)) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int f0 = (blockIdx.x * kFfnWaves + wave) * 16;
  if (f0 >= F) return;
  const size_t row = (size_t)e * F + f0 + (lane & 15);
  const uint16_t *a0 = w_gate + row * d + (lane >> 4) * 8;
  const uint16_t *a1 = w_up + row * d + (lane >> 4) * 8;
  const int ks = k_stagger((blockIdx.y * gridDim.x + blockIdx.x) * kFfnWaves + wave, d);
  constexpr int U4 = U > 2 ? 2 : U;
  for (int c0 = 0; c0 < m; c0 += 16 * kMaxTiles) {
    const int mc = m - c0;
    if (mc <= 16) gateup_tiles<1, U>(a0, a1, h, perm, M, k, d, F, beg, c0, m, f0, ks, act);
    else if (mc <= 32) gateup_tiles<2, U>(a0, a1, h, perm, M, k, d, F, beg, c0, m, f0, ks, act);
    else if (mc <= 64) gateup_tiles<4, U4>(a0, a1, h, perm, M, k, d, F, beg, c0, m, f0, ks, act);
    else gateup_tiles<8, 1>(a0, a1, h, perm, M, k, d, F, beg, c0, m, f0, ks, act);
  }
}

// ---- pass 2 (bf16): down projection, rows scattered to their (token, slot) position -----------
template <int NT, int U>
__device__ __forceinline__ void down_tiles(const uint16_t *a0, const uint16_t *a1, const uint16_t *__restrict__ act,
                                           const int32_t *__restrict__ perm, int M, int k, int d, int F, int beg, int c0,
                                           int m, int j0, int ks, float *__restrict__ y) {
  const int lane = threadIdx.x & 63, col = lane & 15, kg = lane >> 4;
  const uint16_t *bp[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    int p = c0 + j * 16 + col;
    p = p < m ? p : m - 1;
    bp[j] = act + (size_t)pair_index(perm, beg + p, M, k) * F + kg * 8;
  }
  f32x4 acc0[NT], acc1[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) acc0[j] = acc1[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  stream_rows<NT, U>(a0, a1, bp, F, ks, acc0, acc1);
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int p = c0 + j * 16 + col;
    if (p < m) {
      float *dst = y + (size_t)pair_index(perm, beg + p, M, k) * d + j0 + 4 * kg;
      *reinterpret_cast<f32x4 *>(dst) = acc0[j];
      *reinterpret_cast<f32x4 *>(dst + 16) = acc1[j];
    }
  }
}

template <int U>
__global__ __launch_bounds__(kFfnThreads, 2) void ffn_down_bf16_kernel(
    const uint16_t *__restrict__ act, const uint16_t *__restrict__ w_down, const int32_t *__restrict__ seg_expert,
    const int32_t *__restrict__ seg_off, const int32_t *__restrict__ perm, int M, int N, int k, int d, int F,
    float *__restrict__ y) {
  const int seg = blockIdx.y;
  const int e = seg_expert[seg];
  const int beg = seg_off[seg], m = seg_off[seg + 1] - beg;
  if (!segment_ok(e, beg, m, (long long)M * k, N)) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int j0 = (blockIdx.x * kFfnWaves + wave) * 32;
  if (j0 >= d) return;
  const uint16_t *a0 = w_down + ((size_t)e * d + j0 + (lane & 15)) * F + (lane >> 4) * 8;
  const uint16_t *a1 = a0 + (size_t)16 * F;
  const int ks = k_stagger((blockIdx.y * gridDim.x + blockIdx.x) * kFfnWaves + wave, F);
  constexpr int U4 = U > 2 ? 2 : U;
  for (int c0 = 0; c0 < m; c0 += 16 * kMaxTiles) {
    const int mc = m - c0;
    if (mc <= 16) down_tiles<1, U>(a0, a1, act, perm, M, k, d, F, beg, c0, m, j0, ks, y);
    else if (mc <= 32) down_tiles<2, U>(a0, a1, act, perm, M, k, d, F, beg, c0, m, j0, ks, y);
    else if (mc <= 64) down_tiles<4, U4>(a0, a1, act, perm, M, k, d, F, beg, c0, m, j0, ks, y);
    else down_tiles<8, 1>(a0, a1, act, perm, M, k, d, F, beg, c0, m, j0, ks, y);
  }
}

// ---- LDS-tiled bf16 passes (K % 128 == 0) --------------------------------------------------------
// Geometry of one K chunk: U MFMA K-steps of 32 elements; a row of the chunk is RB = 64 U bytes =
// CPR = 4 U pieces of 16 bytes.  Piece c of row r sits at LDS offset r*RB + ((c ^ (r & (CPR-1))) * 16):
// 8 consecutive lanes then touch 8 different 16-byte bank groups both when a row is written
// (lanes along the row) and when it is read in operand layout (lanes across rows).
template <int U>
struct Chunk {
  static constexpr int KC = 32 * U;        // elements per chunk
  static constexpr int CPR = 4 * U;        // 16-byte pieces per row
  static constexpr int RB = 64 * U;        // bytes per row
  static constexpr int RPI = 64 / CPR;     // rows covered by one wave-wide load
  static constexpr int TILE = 16 * RB;     // bytes of a 16-row tile
  static __device__ __forceinline__ int swz(int row, int piece) { return row * RB + ((piece ^ (row & (CPR - 1))) << 4); }
};

// The wave index is taken through readfirstlane in these kernels: it is uniform within a wave, and the
// compiler then keeps everything derived from it (row offsets, tile bases) in scalar registers.
constexpr int kPrefetchTiles = 4;  // walks of up to this many token tiles read their LDS operands one K-step ahead
constexpr int kLdsBytes = 65536;  // 32 KB of wave-private weight tiles + token tile: 2 x (4..16) KB or 1 x 32 KB

// One workgroup pass over K for NT token tiles.  wt0 / wt1: first row of this wave's two 16-row weight
// tiles (row stride K elements).  xbase + xsrc[q] bytes: this lane's source row (already at its 16-byte piece)
// for its q-th share of the token tile.  Accumulates acc0[j] (tile 0) and acc1[j] (tile 1) over the K range
// [kb, kb + kl) of the rows (row stride K).
// make_xsrc(xsrc) fills the token-row offsets from the pair ids the caller has ALREADY loaded into registers; it is
// called after the weight loads of the first chunk have been issued.  Loads complete in issue order, so the wait for
// the (earlier issued) pair ids leaves those weight loads in flight: the expert's first bytes are on their way while
// the token rows are still being looked up.
template <int NT, int U, class XF>
__device__ __forceinline__ void lds_pass(const uint16_t *wt0, const uint16_t *wt1, int K, int kb, int kl, int ks,
                                         const uint16_t *xbase, XF make_xsrc, unsigned char *lds,
                                         f32x4 (&acc0)[NT], f32x4 (&acc1)[NT]) {
  using C = Chunk<U>;
  constexpr int IPW = NT * U / 4;  // token-tile loads per wave per chunk (4 waves share the tile)
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  unsigned char *a_lds = lds + wave * 2 * C::TILE;                 // wave-private: two weight tiles
  unsigned char *x_lds = lds + kFfnWaves * 2 * C::TILE;            // shared: 2 buffers of NT*16 rows
  constexpr int XBUF = NT * 16 * C::RB;
  // two token-tile buffers if they fit beside the weight tiles, else one (and a second barrier per chunk)
  constexpr bool kDoubleX = kFfnWaves * 2 * C::TILE + 2 * XBUF <= kLdsBytes;

  // global -> register staging
  // uniform base + 32-bit byte offset per lane (a tile is 16 rows of at most 2^20 elements): the loads need
  // one offset register each instead of a 64-bit address
  const int lrow = lane / C::CPR, lpc = lane % C::CPR;
  const uint32_t lane_off = 2u * ((uint32_t)lrow * (uint32_t)K + (uint32_t)lpc * 8u);
  bf16x8 GA[2][U], GX[IPW];
  uint32_t xsrc[IPW];
  auto issue_w = [&](int k) {
#pragma unroll
    for (int q = 0; q < U; ++q) {
      const uint32_t off = lane_off + 2u * ((uint32_t)(q * C::RPI) * (uint32_t)K + (uint32_t)k);
      GA[0][q] = ld_stream(at_bytes(wt0, off));
      GA[1][q] = ld_stream(at_bytes(wt1, off));
    }
  };
  auto issue_x = [&](int k) {
#pragma unroll
    for (int q = 0; q < IPW; ++q) GX[q] = ld_frag(at_bytes(xbase, xsrc[q] + 2u * (uint32_t)k));
  };
  auto issue = [&](int k) {
    issue_w(k);
    issue_x(k);
  };
  auto park = [&](int buf) {
#pragma unroll
    for (int q = 0; q < U; ++q) {
      const int row = q * C::RPI + lrow;
      *reinterpret_cast<bf16x8 *>(a_lds + C::swz(row, lpc)) = GA[0][q];
      *reinterpret_cast<bf16x8 *>(a_lds + C::TILE + C::swz(row, lpc)) = GA[1][q];
    }
#pragma unroll
    for (int q = 0; q < IPW; ++q) {
      const int g = (wave * IPW + q) * 64 + lane;
      *reinterpret_cast<bf16x8 *>(x_lds + buf * XBUF + C::swz(g / C::CPR, g % C::CPR)) = GX[q];
    }
  };
  const int r = lane & 15, kg = lane >> 4;
  // Up to kPrefetchTiles token tiles: the operands of K-step u + 1 are read from LDS into a second register set
  // before the matrix instructions of step u are issued, so that the LDS latency of a step is covered by the
  // previous step's MFMAs (the scheduling barriers keep the compiler from sinking the reads back to their uses).
  // With 8 token tiles the registers do not hold a second set and the reads stay next to their uses (measured:
  // issuing all reads of a step first is 2-4 % slower there).
  auto compute = [&](int buf) {
    if constexpr (NT <= kPrefetchTiles) {
      bf16x8 fa0[2], fa1[2], fb[2][NT];
      auto fetch = [&](int u) {
        const int pc = 4 * u + kg, st = u & 1;
        fa0[st] = *reinterpret_cast<const bf16x8 *>(a_lds + C::swz(r, pc));
        fa1[st] = *reinterpret_cast<const bf16x8 *>(a_lds + C::TILE + C::swz(r, pc));
#pragma unroll
        for (int j = 0; j < NT; ++j)
          fb[st][j] = *reinterpret_cast<const bf16x8 *>(x_lds + buf * XBUF + C::swz(16 * j + r, pc));
      };
      fetch(0);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (u + 1 < U) fetch(u + 1);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          acc0[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa0[u & 1], fb[u & 1][j], acc0[j], 0, 0, 0);
          acc1[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa1[u & 1], fb[u & 1][j], acc1[j], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int pc = 4 * u + kg;
        const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(a_lds + C::swz(r, pc));
        const bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(a_lds + C::TILE + C::swz(r, pc));
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          const bf16x8 b = *reinterpret_cast<const bf16x8 *>(x_lds + buf * XBUF + C::swz(16 * j + r, pc));
          acc0[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, b, acc0[j], 0, 0, 0);
          acc1[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, b, acc1[j], 0, 0, 0);
        }
      }
    }
  };

  // the walk covers the elements [kb, kb + kl) of every row (kl a multiple of the chunk), starting
  // ks elements into that range and wrapping inside it
  const int nst = kl / C::KC;
  int k = ((ks % kl) / C::KC) * C::KC;
  issue_w(kb + k);
  __builtin_amdgcn_sched_barrier(0);  // keep the weight loads ahead of the wait for the pair ids
  make_xsrc(xsrc);
  issue_x(kb + k);
  for (int i = 0; i < nst; ++i) {
    park(kDoubleX ? (i & 1) : 0);
    k += C::KC;
    k = k >= kl ? k - kl : k;
    if (i + 1 < nst) issue(kb + k);
    __syncthreads();  // token tile i complete; also orders this wave's tile writes before its reads
    compute(kDoubleX ? (i & 1) : 0);
    if (!kDoubleX) __syncthreads();  // everybody has read the single token tile before it is overwritten
  }
  __syncthreads();  // the LDS tiles may be reused by the caller's next pass
}

// The workgroup's work item derived on the spot (fused layer, small trees).  shortlist[r] = expert with
// rank r in the shortlist (descending aggregate score, which is also roughly descending segment size),
// rank_count[r] = number of its surviving pairs, tok_ids = restricted routing table [M, k].  The work items
// are the pieces (piece_count per expert) of the shortlisted experts in rank order; the workgroup takes the
// one that xcd_map assigns to it and collects that piece's pairs in token order into plist (LDS,
// kPiecePairs entries).  The tables are read in one round of independent loads per 256 tokens.
// Requires B <= kFfnThreads, k <= kSelfMaxK, M <= kSelfMaxTokens.  misc: 8 int32 of LDS scratch.
// Called by every thread of the workgroup (it synchronises).  Returns the expert (-1: no work item) and the
// number of work items.
constexpr int kSelfMaxK = 16;
// lists != NULL (the fused prologue has already written every shortlist rank's pairs, rank r at
// lists + r * list_stride): nothing is collected, list receives the address of the piece inside that table.
__device__ __forceinline__ int self_segment(const int32_t *__restrict__ rank_count,
                                            const int32_t *__restrict__ shortlist, int B,
                                            const int32_t *__restrict__ tok_ids, int M, int k, int tiles,
                                            int32_t *misc, int32_t *plist, int &m, int &item, int &tile,
                                            int &n_items, const int32_t *__restrict__ lists, int list_stride,
                                            const int32_t *&list) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int ids[kSelfMaxK];
  auto load_ids = [&](int t) {
#pragma unroll
    for (int j = 0; j < kSelfMaxK; ++j) ids[j] = (j < k && t < M) ? tok_ids[(size_t)t * k + j] : -1;
  };
  list = plist;
  if (!lists) load_ids(tid);
  const int c = tid < B ? rank_count[tid] : 0;
  const int ex = tid < B ? shortlist[tid] : -1;
  const int q = c > 0 ? piece_count(c) : 0;
  int incl = q;  // inclusive scan of the piece counts over the shortlist ranks
#pragma unroll
  for (int sft = 1; sft < kWave; sft <<= 1) {
    const int v = __shfl_up(incl, sft, kWave);
    if (lane >= sft) incl += v;
  }
  if (lane == kWave - 1) misc[1 + wave] = incl;
  if (tid == 0) misc[0] = -1;
  __syncthreads();
  int before = 0;
  n_items = 0;
  for (int w = 0; w < kFfnWaves; ++w) {
    if (w < wave) before += misc[1 + w];
    n_items += misc[1 + w];
  }
  const bool has_work = xcd_map(tiles, n_items, item, tile);
  const int first = before + incl - q;  // first work item of this thread's expert
  if (has_work && item >= first && item < first + q) {  // one thread at most
    const int len = (c + q - 1) / q, p = item - first;
    misc[0] = ex;
    misc[5] = p * len;                 // the piece: pairs [lo, lo + m) of the expert's segment
    misc[6] = min(len, c - p * len);
    misc[7] = tid;                     // its shortlist rank
  }
  __syncthreads();
  const int e = misc[0];
  m = 0;
  if (e < 0) return -1;
  const int lo = misc[5];
  m = misc[6];
  if (lists) {
    list = lists + (size_t)misc[7] * list_stride + lo;
    return e;
  }
  int base = 0;
  for (int t0 = 0; t0 < M && base < lo + m; t0 += kFfnThreads) {  // uniform trip count
    const int t = t0 + tid;
    if (t0 > 0) load_ids(t);
    int slot = -1;
#pragma unroll
    for (int j = 0; j < kSelfMaxK; ++j)
      if (ids[j] == e) slot = j;
    const unsigned long long mask = __ballot(slot >= 0);
    __syncthreads();  // everybody has read the wave counts of the previous round
    if (lane == 0) misc[1 + wave] = __popcll(mask);
    __syncthreads();
    int pos = base;
    for (int w = 0; w < wave; ++w) pos += misc[1 + w];
    pos += __popcll(mask & ((1ull << lane) - 1ull)) - lo;
    if (slot >= 0 && pos >= 0 && pos < m) plist[pos] = t * k + slot;
    for (int w = 0; w < kFfnWaves; ++w) base += misc[1 + w];
  }
  __syncthreads();
  return e;
}

// plist: the segment's pairs (flat ids t * k + slot, tokens ascending), in global memory or LDS; n_pairs = M * k.
__device__ __forceinline__ int pair_at(const int32_t *plist, int p, int n_pairs) {
  const int q = plist[p];
  return q < 0 ? 0 : (q >= n_pairs ? n_pairs - 1 : q);
}

template <int NT, int U>
__device__ __forceinline__ void gateup_lds(const uint16_t *wt0, const uint16_t *wt1, const uint16_t *__restrict__ h,
                                           const int32_t *plist, int n_pairs, int k, int d, int F, int c0, int m,
                                           int f0, int ks, unsigned char *lds, uint16_t *__restrict__ act) {
  using C = Chunk<U>;
  constexpr int IPW = NT * U / 4;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int pair[IPW];  // this lane's pair ids, loaded now and turned into row offsets inside lds_pass
#pragma unroll
  for (int q = 0; q < IPW; ++q) {
    const int g = (wave * IPW + q) * 64 + lane;
    int p = c0 + g / C::CPR;
    p = p < m ? p : m - 1;  // pad rows repeat the last token; their columns are never stored
    pair[q] = plist[p];
  }
  // 32-bit byte offsets: M * d < 2^31 elements (checked on the host)
  auto make_xsrc = [&](uint32_t (&xsrc)[IPW]) {
#pragma unroll
    for (int q = 0; q < IPW; ++q) {
      const int g = (wave * IPW + q) * 64 + lane;
      const int pr = pair[q] < 0 ? 0 : (pair[q] >= n_pairs ? n_pairs - 1 : pair[q]);
      xsrc[q] = 2u * ((uint32_t)(pr / k) * (uint32_t)d + (uint32_t)(g % C::CPR) * 8u);
    }
  };
  f32x4 accg[NT], accu[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) accg[j] = accu[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  lds_pass<NT, U>(wt0, wt1, d, 0, d, ks, h, make_xsrc, lds, accg, accu);
  const int col = lane & 15, kg = lane >> 4;
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int p = c0 + j * 16 + col;
    if (p < m) {
      uint16_t o[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = float_to_bf16_bits(silu_f(accg[j][i]) * accu[j][i]);
      uint2 pk;
      pk.x = (uint32_t)o[0] | ((uint32_t)o[1] << 16);
      pk.y = (uint32_t)o[2] | ((uint32_t)o[3] << 16);
      *reinterpret_cast<uint2 *>(act + (size_t)pair_at(plist, p, n_pairs) * F + f0 + 4 * kg) = pk;
    }
  }
}

// rank_count != NULL: self-segmenting mode (items / perm unused; n_seg = B); otherwise items + perm.
__global__ __launch_bounds__(kFfnThreads, 2) void ffn_gateup_lds_kernel(
    const uint16_t *__restrict__ h, const uint16_t *__restrict__ w_gate, const uint16_t *__restrict__ w_up,
    const int4 *__restrict__ items, const int32_t *__restrict__ perm, const int32_t *__restrict__ rank_count,
    const int32_t *__restrict__ shortlist, const int32_t *__restrict__ tok_ids, int n_seg, int cap, int M, int N,
    int k, int d, int F, long long perm_len, int4 *__restrict__ pub_items, int32_t *__restrict__ pub_lists,
    const int32_t *__restrict__ lists, int list_stride, uint16_t *__restrict__ act) {
  __shared__ __align__(16) unsigned char lds[kLdsBytes];
  __shared__ int32_t own_pairs[kPiecePairs];
  __shared__ int32_t misc[8];
  const int tiles = (F / 16 + kFfnWaves - 1) / kFfnWaves;
  int tile, rank, e, m;
  const int32_t *plist;
  if (rank_count) {
    int n_items;
    e = self_segment(rank_count, shortlist, n_seg, tok_ids, M, k, tiles, misc, own_pairs, m, rank, tile, n_items,
                     lists, list_stride, plist);
    // The work items found here are published for the down pass (same table format as the budget stage's):
    // workgroup 0 writes the count, the first row tile of every item its entry and its pair list.
    if (pub_items && blockIdx.x == 0 && threadIdx.x == 0) pub_items[0] = int4{n_items, 0, 0, 0};
    if (e < 0 || e >= N || m <= 0 || m > kPiecePairs) return;
    if (pub_items && tile == 0) {
      for (int p = threadIdx.x; p < m; p += kFfnThreads) pub_lists[(size_t)rank * kPiecePairs + p] = own_pairs[p];
      if (threadIdx.x == 0) pub_items[1 + rank] = int4{rank, e, rank * kPiecePairs, m};
    }
  } else {
    const int4 it = xcd_item(tiles, cap, items, tile, rank);
    e = it.y;
    m = it.w;
    if (it.x < 0 || !segment_ok(e, it.z, m, perm_len, N)) return;
    plist = perm + it.z;
  }
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // F is a multiple of 32 but a workgroup covers 64 gate rows: the waves of a last, partial workgroup
  // redo rows of the previous tile (same values, same destination) so that every wave reaches the barriers.
  int f0 = (tile * kFfnWaves + wave) * 16;
  f0 = f0 < F ? f0 : F - 16;
  const uint16_t *wt0 = w_gate + ((size_t)e * F + f0) * d;
  const uint16_t *wt1 = w_up + ((size_t)e * F + f0) * d;
  const int ks = k_stagger(rank, d);
  const int n_pairs = M * k;
  for (int c0 = 0; c0 < m; c0 += 16 * kMaxTiles) {
    const int mc = m - c0;
    if (mc <= 16) gateup_lds<1, 4>(wt0, wt1, h, plist, n_pairs, k, d, F, c0, m, f0, ks, lds, act);
    else if (mc <= 32) gateup_lds<2, 4>(wt0, wt1, h, plist, n_pairs, k, d, F, c0, m, f0, ks, lds, act);
    else if (mc <= 64) gateup_lds<4, 4>(wt0, wt1, h, plist, n_pairs, k, d, F, c0, m, f0, ks, lds, act);
    else gateup_lds<8, 4>(wt0, wt1, h, plist, n_pairs, k, d, F, c0, m, f0, ks, lds, act);
  }
}

template <int NT, int U>
__device__ __forceinline__ void down_lds(const uint16_t *wt0, const uint16_t *wt1, const uint16_t *__restrict__ act,
                                         const int32_t *plist, int n_pairs, int d, int F, int kb, int kl, int c0, int m,
                                         int j0, int ks, unsigned char *lds, float *__restrict__ y) {
  using C = Chunk<U>;
  constexpr int IPW = NT * U / 4;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int pair[IPW];  // this lane's pair ids, loaded now and turned into row offsets inside lds_pass
#pragma unroll
  for (int q = 0; q < IPW; ++q) {
    const int g = (wave * IPW + q) * 64 + lane;
    int p = c0 + g / C::CPR;
    p = p < m ? p : m - 1;
    pair[q] = plist[p];
  }
  // 32-bit byte offsets: M * k * F < 2^31 elements (checked on the host)
  auto make_xsrc = [&](uint32_t (&xsrc)[IPW]) {
#pragma unroll
    for (int q = 0; q < IPW; ++q) {
      const int g = (wave * IPW + q) * 64 + lane;
      const int pr = pair[q] < 0 ? 0 : (pair[q] >= n_pairs ? n_pairs - 1 : pair[q]);
      xsrc[q] = 2u * ((uint32_t)pr * (uint32_t)F + (uint32_t)(g % C::CPR) * 8u);
    }
  };
  f32x4 acc0[NT], acc1[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) acc0[j] = acc1[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  lds_pass<NT, U>(wt0, wt1, F, kb, kl, ks, act, make_xsrc, lds, acc0, acc1);
  const int col = lane & 15, kg = lane >> 4;
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int p = c0 + j * 16 + col;
    if (p < m) {
      float *dst = y + (size_t)pair_at(plist, p, n_pairs) * d + j0 + 4 * kg;
      *reinterpret_cast<f32x4 *>(dst) = acc0[j];
      *reinterpret_cast<f32x4 *>(dst + 16) = acc1[j];
    }
  }
}

__global__ __launch_bounds__(kFfnThreads, 2) void ffn_down_lds_kernel(
    const uint16_t *__restrict__ act, const uint16_t *__restrict__ w_down, const int4 *__restrict__ items,
    const int32_t *__restrict__ perm, const int32_t *__restrict__ rank_count, const int32_t *__restrict__ shortlist,
    const int32_t *__restrict__ tok_ids, int n_seg, int cap, int M, int N, int k, int d, int F, int splits,
    long long perm_len, const int32_t *__restrict__ lists, int list_stride, float *__restrict__ y) {
  __shared__ __align__(16) unsigned char lds[kLdsBytes];
  __shared__ int32_t own_pairs[kPiecePairs];
  __shared__ int32_t misc[8];
  // a work item is (row tile, K split): split sp sums the 128-element chunks [sp n / splits, (sp + 1) n / splits)
  // of F into its own copy of y, which the combine adds up in split order
  const int tiles = ((d / 32 + kFfnWaves - 1) / kFfnWaves) * splits;
  int tile, rank, e, m;
  const int32_t *plist;
  if (rank_count) {
    int n_items;
    e = self_segment(rank_count, shortlist, n_seg, tok_ids, M, k, tiles, misc, own_pairs, m, rank, tile, n_items,
                     lists, list_stride, plist);
    if (e < 0 || e >= N || m <= 0 || m > kPiecePairs) return;
  } else {
    const int4 it = xcd_item(tiles, cap, items, tile, rank);
    e = it.y;
    m = it.w;
    if (it.x < 0 || !segment_ok(e, it.z, m, perm_len, N)) return;
    plist = perm + it.z;
  }
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int sp = tile % splits;
  tile /= splits;
  int j0 = (tile * kFfnWaves + wave) * 32;
  j0 = j0 < d ? j0 : d - 32;  // see ffn_gateup_lds_kernel
  const uint16_t *wt0 = w_down + ((size_t)e * d + j0) * F;
  const uint16_t *wt1 = wt0 + (size_t)16 * F;
  const int nch = F / 128, kb = (int)((long long)sp * nch / splits) * 128;
  const int kl = (int)((long long)(sp + 1) * nch / splits) * 128 - kb;
  const int ks = k_stagger(rank + sp, kl);
  const int n_pairs = M * k;
  y += (size_t)sp * n_pairs * d;
  for (int c0 = 0; c0 < m; c0 += 16 * kMaxTiles) {
    const int mc = m - c0;
    if (mc <= 16) down_lds<1, 4>(wt0, wt1, act, plist, n_pairs, d, F, kb, kl, c0, m, j0, ks, lds, y);
    else if (mc <= 32) down_lds<2, 4>(wt0, wt1, act, plist, n_pairs, d, F, kb, kl, c0, m, j0, ks, lds, y);
    else if (mc <= 64) down_lds<4, 4>(wt0, wt1, act, plist, n_pairs, d, F, kb, kl, c0, m, j0, ks, lds, y);
    else down_lds<8, 4>(wt0, wt1, act, plist, n_pairs, d, F, kb, kl, c0, m, j0, ks, lds, y);
  }
}

// ---- fp32 path: one wave per weight row, lanes stride K (correctness path for small layers) ----
__global__ __launch_bounds__(kFfnThreads) void ffn_gateup_f32_kernel(
    const float *__restrict__ h, const float *__restrict__ w_gate, const float *__restrict__ w_up,
    const int32_t *__restrict__ seg_expert, const int32_t *__restrict__ seg_off, const int32_t *__restrict__ perm,
    int M, int N, int k, int d, int F, float *__restrict__ act) {
  const int seg = blockIdx.y;
  const int e = seg_expert[seg];
  const int beg = seg_off[seg], m = seg_off[seg + 1] - beg;
  if (!segment_ok(e, beg, m, (long long)M * k, N)) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int f = blockIdx.x * kFfnWaves + wave;
  if (f >= F) return;
  const float *wg = w_gate + ((size_t)e * F + f) * d;
  const float *wu = w_up + ((size_t)e * F + f) * d;
  for (int p = 0; p < m; ++p) {
    const float *x = h + (size_t)(pair_index(perm, beg + p, M, k) / k) * d;
    float g = 0.f, u = 0.f;
    for (int j = lane; j < d; j += kWave) {
      const float xv = x[j];
      g = fmaf(wg[j], xv, g);
      u = fmaf(wu[j], xv, u);
    }
    g = wave_sum(g);
    u = wave_sum(u);
    if (lane == 0) act[(size_t)(beg + p) * F + f] = g / (1.0f + expf(-g)) * u;
  }
}

__global__ __launch_bounds__(kFfnThreads) void ffn_down_f32_kernel(
    const float *__restrict__ act, const float *__restrict__ w_down, const int32_t *__restrict__ seg_expert,
    const int32_t *__restrict__ seg_off, const int32_t *__restrict__ perm, int M, int N, int k, int d, int F,
    float *__restrict__ y) {
  const int seg = blockIdx.y;
  const int e = seg_expert[seg];
  const int beg = seg_off[seg], m = seg_off[seg + 1] - beg;
  if (!segment_ok(e, beg, m, (long long)M * k, N)) return;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int j = blockIdx.x * kFfnWaves + wave;
  if (j >= d) return;
  const float *wd = w_down + ((size_t)e * d + j) * F;
  for (int p = 0; p < m; ++p) {
    const float *a = act + (size_t)(beg + p) * F;
    float acc = 0.f;
    for (int f = lane; f < F; f += kWave) acc = fmaf(wd[f], a[f], acc);
    acc = wave_sum(acc);
    if (lane == 0) y[(size_t)pair_index(perm, beg + p, M, k) * d + j] = acc;
  }
}

// ---- combine: out[t] = residual[t] + sum over surviving slots (slot order) of w * y[t*k+slot] ---
// Four consecutive outputs per thread; y holds `splits` partial copies split_stride floats apart (K-split
// down pass).  The rows of dropped slots hold stale scratch: they are loaded
// (valid memory) but never enter the sum.
// the four outputs j .. j+3 of token t (before storage rounding)
template <typename T>
__device__ __forceinline__ f32x4 combine_four(const float *__restrict__ y, const int32_t *__restrict__ tok_ids,
                                              const float *__restrict__ tok_w, const T *__restrict__ residual, int t,
                                              int j, int k, int d, int splits, size_t split_stride) {
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if (residual) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = Elem<T>::load(residual + (size_t)t * d + j + i);
  }
  const float *yt = y + (size_t)t * k * d + j;
  const int32_t *ids = tok_ids + (size_t)t * k;
  const float *wt = tok_w + (size_t)t * k;
  // a pair's row is the sum of its K-split copies, added in split order
  auto row = [&](const float *p) {
    f32x4 v = *reinterpret_cast<const f32x4 *>(p);
    for (int sp = 1; sp < splits; ++sp) v += *reinterpret_cast<const f32x4 *>(p + sp * split_stride);
    return v;
  };
  int s = 0;
  for (; s + 4 <= k; s += 4) {
    f32x4 v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = row(yt + (size_t)(s + u) * d);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (ids[s + u] >= 0) {
        const float w = wt[s + u];
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = fmaf(w, v[u][i], acc[i]);
      }
    }
  }
  for (; s < k; ++s) {
    if (ids[s] >= 0) {
      const f32x4 v = row(yt + (size_t)s * d);
      const float w = wt[s];
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = fmaf(w, v[i], acc[i]);
    }
  }
  return acc;
}

template <typename T>
__global__ __launch_bounds__(256) void combine_kernel(const float *__restrict__ y, const int32_t *__restrict__ tok_ids,
                                                      const float *__restrict__ tok_w, const T *__restrict__ residual,
                                                      int k, int d, int splits, size_t split_stride,
                                                      T *__restrict__ out) {
  const int t = blockIdx.y;
  const int j = (blockIdx.x * blockDim.x + threadIdx.x) * 4;
  if (j >= d) return;
  const f32x4 acc = combine_four<T>(y, tok_ids, tok_w, residual, t, j, k, d, splits, split_stride);
#pragma unroll
  for (int i = 0; i < 4; ++i) Elem<T>::store(out + (size_t)t * d + j + i, acc[i]);
}

// The combine of a layer inside a stack that scales its layer inputs: one workgroup per token writes the row of the
// new hidden state and, from the STORED (rounded) values, the next layer's input x = row / rms(row) - with the
// element-to-thread mapping and summation order of rms_scale_row, so that the result equals, bit for bit, what
// rms_scale_kernel makes of the stored row.  d <= 8192: a thread holds up to 8 outputs.
template <typename T>
__global__ __launch_bounds__(kRmsThreads) void combine_scale_kernel(const float *__restrict__ y,
                                                                    const int32_t *__restrict__ tok_ids,
                                                                    const float *__restrict__ tok_w,
                                                                    const T *__restrict__ residual, int k, int d,
                                                                    int splits, size_t split_stride,
                                                                    T *__restrict__ out, T *__restrict__ x_next) {
  __shared__ float part[kRmsThreads];
  const int t = blockIdx.x, tid = threadIdx.x;
  float v[kRmsChunks][4];
#pragma unroll
  for (int c = 0; c < kRmsChunks; ++c) {
    const int j = (c * kRmsThreads + tid) * 4;
    if (j < d) {
      const f32x4 acc = combine_four<T>(y, tok_ids, tok_w, residual, t, j, k, d, splits, split_stride);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        Elem<T>::store(out + (size_t)t * d + j + i, acc[i]);
        v[c][i] = Elem<T>::stored(acc[i]);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) v[c][i] = 0.f;
    }
  }
  const float scale = rms_scale_of_row(v, d, part);
#pragma unroll
  for (int c = 0; c < kRmsChunks; ++c) {
    const int j = (c * kRmsThreads + tid) * 4;
    if (j < d)
#pragma unroll
      for (int i = 0; i < 4; ++i) Elem<T>::store(x_next + (size_t)t * d + j + i, v[c][i] * scale);
  }
}

template <int U>
static hipError_t launch_bf16(const moespec_desc &ds, const moespec_weights &wt, const void *h, int M, int n_seg,
                              const int32_t *seg_expert, const int32_t *seg_off, const int32_t *perm, void *act,
                              float *y, int pass, hipStream_t st) {
  const int d = ds.d, F = ds.d_ff, k = ds.top_k;
  if (pass == 1) {
    dim3 grid((F / 16 + kFfnWaves - 1) / kFfnWaves, n_seg);
    ffn_gateup_bf16_kernel<U><<<grid, kFfnThreads, 0, st>>>(
        static_cast<const uint16_t *>(h), static_cast<const uint16_t *>(wt.w_gate),
        static_cast<const uint16_t *>(wt.w_up), seg_expert, seg_off, perm, M, ds.n_experts, k, d, F,
        static_cast<uint16_t *>(act));
  } else {
    dim3 grid((d / 32 + kFfnWaves - 1) / kFfnWaves, n_seg);
    ffn_down_bf16_kernel<U><<<grid, kFfnThreads, 0, st>>>(static_cast<const uint16_t *>(act),
                                                          static_cast<const uint16_t *>(wt.w_down), seg_expert,
                                                          seg_off, perm, M, ds.n_experts, k, d, F, y);
  }
  return hipGetLastError();
}

// The self-segmenting mode needs both passes on the LDS-tiled kernels and a tree small enough for
// their LDS scratch.
bool expert_ffn_self_segmenting(const moespec_desc &ds, int M) {
  return ds.dtype == MOESPEC_BF16 && ds.d % 128 == 0 && ds.d_ff % 128 == 0 && ds.n_experts <= kSelfMaxExperts &&
         M <= kSelfMaxTokens && ds.top_k <= kSelfMaxK;
}

// K-split of the LDS-tiled down pass: when its (segment, row tile) items alone cannot give every compute
// unit two workgroups, each item is cut along F into up to kMaxDownSplits parts with their own copy of y,
// as long as a part keeps at least 16 chunks (shorter walks are dominated by their start-up: measured
// slower at F = 1024, 1.6x to 2.7x faster at F = 14336 with 4 or 2 loaded experts).
int down_splits(const moespec_desc &ds, int n_seg) {
  int splits = 1;
  if (ds.dtype == MOESPEC_BF16 && ds.d_ff % 128 == 0) {
    const int tiles = (ds.d / 32 + kFfnWaves - 1) / kFfnWaves;
    while (splits < kMaxDownSplits && (long long)n_seg * tiles * splits * 2 <= 512 && ds.d_ff / 128 >= 32 * splits)
      splits *= 2;
  }
  return splits;
}

static int pick_unroll(int K) { return K % 128 == 0 ? 4 : (K % 64 == 0 ? 2 : 1); }

hipError_t launch_expert_ffn(const moespec_desc &ds, const moespec_weights &wt, const void *h, int M, int n_seg,
                             const int32_t *seg_expert, const int32_t *seg_off, const int32_t *perm,
                             const int32_t *tok_ids, const float *tok_w, const void *residual, void *out, void *act,
                             float *y, int4 *items, bool items_ready, const int32_t *rank_count,
                             const int32_t *shortlist, int4 *pub_items, int32_t *pub_lists, hipStream_t st,
                             void *const *trace, const int32_t *lists, int list_stride, void *x_next) {
  const int d = ds.d, F = ds.d_ff, k = ds.top_k;
  hipError_t e;
  if (lists) pub_items = nullptr;  // every pass reads the prologue's lists: nothing to publish
  if (rank_count && !(shortlist && expert_ffn_self_segmenting(ds, M) && n_seg <= kFfnThreads)) rank_count = nullptr;
  if (!rank_count && !items_ready && !items) return hipErrorInvalidValue;
  const int cap = items_capacity(n_seg, M, k);  // work items of the LDS-tiled passes
  if (ds.dtype == MOESPEC_BF16 && !rank_count && !items_ready && (d % 128 == 0 || F % 128 == 0)) {
    segment_items_kernel<<<1, 256, 0, st>>>(seg_expert, seg_off, n_seg, M, k, cap, items);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  auto mark = [&](int i) {
    if (trace && trace[i]) (void)hipEventRecord(static_cast<hipEvent_t>(trace[i]), st);
  };
  const int splits = down_splits(ds, n_seg);
  const bool publish = rank_count && pub_items && pub_lists;
  const size_t split_stride = (size_t)M * k * d;
  if (ds.dtype == MOESPEC_BF16) {
    for (int pass = 1; pass <= 2; ++pass) {
      if ((pass == 1 ? d : F) % 128 == 0) {
        if (pass == 1) {
          const int grid = xcd_grid((F / 16 + kFfnWaves - 1) / kFfnWaves, cap);
          ffn_gateup_lds_kernel<<<grid, kFfnThreads, 0, st>>>(
              static_cast<const uint16_t *>(h), static_cast<const uint16_t *>(wt.w_gate),
              static_cast<const uint16_t *>(wt.w_up), items, perm, rank_count, shortlist, tok_ids, n_seg, cap, M,
              ds.n_experts, k, d, F, (long long)M * k, publish ? pub_items : nullptr, pub_lists,
              rank_count ? lists : nullptr, list_stride, static_cast<uint16_t *>(act));
        } else {
          const int grid = xcd_grid(((d / 32 + kFfnWaves - 1) / kFfnWaves) * splits, cap);
          // after a self-segmenting gate/up pass the down pass reads the segments that pass has published
          ffn_down_lds_kernel<<<grid, kFfnThreads, 0, st>>>(
              static_cast<const uint16_t *>(act), static_cast<const uint16_t *>(wt.w_down),
              publish ? pub_items : items, publish ? pub_lists : perm, publish ? nullptr : rank_count, shortlist,
              tok_ids, n_seg, cap, M, ds.n_experts, k, d, F, splits,
              publish ? (long long)cap * kPiecePairs : (long long)M * k, rank_count ? lists : nullptr, list_stride, y);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
        mark(pass - 1);
        continue;
      }
      switch (pick_unroll(pass == 1 ? d : F)) {
        case 4: e = launch_bf16<4>(ds, wt, h, M, n_seg, seg_expert, seg_off, perm, act, y, pass, st); break;
        case 2: e = launch_bf16<2>(ds, wt, h, M, n_seg, seg_expert, seg_off, perm, act, y, pass, st); break;
        default: e = launch_bf16<1>(ds, wt, h, M, n_seg, seg_expert, seg_off, perm, act, y, pass, st); break;
      }
      if (e != hipSuccess) return e;
      mark(pass - 1);
    }
    if (!out) return hipSuccess;  // the caller only wants the per-pair outputs y
    if (x_next) {
      combine_scale_kernel<uint16_t><<<M, kRmsThreads, 0, st>>>(y, tok_ids, tok_w, static_cast<const uint16_t *>(residual),
                                                              k, d, splits, split_stride, static_cast<uint16_t *>(out),
                                                              static_cast<uint16_t *>(x_next));
    } else {
      dim3 cgrid((d / 4 + 255) / 256, M);
      combine_kernel<uint16_t><<<cgrid, 256, 0, st>>>(y, tok_ids, tok_w, static_cast<const uint16_t *>(residual), k, d,
                                                      splits, split_stride, static_cast<uint16_t *>(out));
    }
    e = hipGetLastError();
    mark(2);
    return e;
  }
  dim3 g1((F + kFfnWaves - 1) / kFfnWaves, n_seg);
  ffn_gateup_f32_kernel<<<g1, kFfnThreads, 0, st>>>(static_cast<const float *>(h),
                                                    static_cast<const float *>(wt.w_gate),
                                                    static_cast<const float *>(wt.w_up), seg_expert, seg_off, perm, M,
                                                    ds.n_experts, k, d, F, static_cast<float *>(act));
  if ((e = hipGetLastError()) != hipSuccess) return e;
  mark(0);
  dim3 g2((d + kFfnWaves - 1) / kFfnWaves, n_seg);
  ffn_down_f32_kernel<<<g2, kFfnThreads, 0, st>>>(static_cast<const float *>(act),
                                                  static_cast<const float *>(wt.w_down), seg_expert, seg_off, perm, M,
                                                  ds.n_experts, k, d, F, y);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  mark(1);
  if (!out) return hipSuccess;
  if (x_next) {
    combine_scale_kernel<float><<<M, kRmsThreads, 0, st>>>(y, tok_ids, tok_w, static_cast<const float *>(residual), k, d,
                                                         1, split_stride, static_cast<float *>(out),
                                                         static_cast<float *>(x_next));
  } else {
    dim3 cgrid((d / 4 + 255) / 256, M);
    combine_kernel<float><<<cgrid, 256, 0, st>>>(y, tok_ids, tok_w, static_cast<const float *>(residual), k, d, 1,
                                                 split_stride, static_cast<float *>(out));
  }
  e = hipGetLastError();
  mark(2);
  return e;
}

}  // namespace moespec
