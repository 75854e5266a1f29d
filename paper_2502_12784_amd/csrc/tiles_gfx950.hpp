// Tile-level building blocks shared by the attention kernels on gfx950: work-item mapping,
// swizzled LDS tiles, global -> LDS movement, transposed accumulator stores.
#pragma once
#include "mma_gfx950.hpp"

namespace spark {

// Workgroups are handed to the 8 XCDs round-robin by linear id.  Map the id so that each XCD
// gets one contiguous range of logical work items: the query tiles of one head then share
// that XCD's L2 for K and V.
static __device__ __forceinline__ int xcd_contiguous(int id, int total) {
  const int per = total >> 3, rem = total & 7;
  const int xcd = id & 7, slot = id >> 3;
  const int base = xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per;
  return base + slot;
}

// Where one [B, H, N, d] tensor lives: element strides of the batch, head and row (sequence)
// indices; the d elements of a row are contiguous.  [B,H,N,d] contiguous is {H*N*d, N*d, d};
// a [B,N,H,d] buffer viewed as [B,H,N,d] is {N*H*d, d, H*d}.
struct TensorMap {
  long long batch, head, row;
};
// Element offset of (batch, head) = flat index `bh` of B*H.
static __device__ __forceinline__ size_t head_base(const TensorMap& m, int bh, int H) {
  const int b = bh / H, h = bh - b * H;
  return (size_t)b * (size_t)m.batch + (size_t)h * (size_t)m.head;
}
// Bytes a buffer view of one head must span: rows 0..n-1, the last one dh elements long.
static __device__ __forceinline__ uint32_t head_span_bytes(const TensorMap& m, int n, int dh) {
  return (uint32_t)(((size_t)(n - 1) * (size_t)m.row + (size_t)dh) * 2);
}

// Head dimensions below the tile width.  The kernels are compiled for rows of D = 64 or 128
// elements; a head dimension dh < D (a multiple of 8) runs in the next wider one with the columns
// dh..D-1 of every operand read as zeros (they add nothing to any contraction) and never stored.
// A fragment load of 8 elements starting at column `col`:
template <typename V8, typename T>
static __device__ __forceinline__ V8 load_row_chunk(const T* row, int col, int dh) {
  V8 z;
#pragma unroll
  for (int i = 0; i < 8; ++i) z[i] = (T)0.f;
  return col < dh ? *reinterpret_cast<const V8*>(row + col) : z;
}

// Work items per head for a kernel that walks `tiles` tiles: causal kernels pair tile p with
// tile tiles-1-p.
template <bool CAUSAL>
static __host__ __device__ __forceinline__ int causal_items(int tiles) {
  return CAUSAL ? (tiles + 1) / 2 : tiles;
}

// ---------------------------------------------------------------------------------------
// Swizzled LDS tiles.  A tile that is read both row-wise (16 bytes of one row per lane: A/B
// operands contracted over d) and transposed (ds_read_b64_tr_b16 over 4 rows x 64 bytes)
// cannot be made conflict-free by padding alone, so rows are unpadded (2*D bytes) and the
// 16-byte chunk index is XORed with a function of the row:
//   D = 128 (16 chunks/row):  f(r) = ((r & 3) << 2) | ((r >> 2) & 3)
//   D =  64 ( 8 chunks/row):  x = (r >> 1) & 7,  f = ((x & 1) << 2) | ((x >> 1) & 3)
// 16 consecutive rows at one logical chunk then fall into 16 different 16-byte bank groups,
// and the 4 rows x 4 chunks of a transposing read into 16 different ones as well.  f depends
// on r mod 16 only, so per-lane offsets are computed once and every tile / sub-tile / k-step
// displacement is an immediate.
// ---------------------------------------------------------------------------------------
template <int D>
static __device__ __forceinline__ int swz(int row) {
  if (D == 128) return ((row & 3) << 2) | ((row >> 2) & 3);
  const int x = (row >> 1) & 7;
  return ((x & 1) << 2) | ((x >> 1) & 3);
}
template <int D>
static __device__ __forceinline__ int swz_off(int row, int chunk) {
  return row * (2 * D) + ((chunk ^ swz<D>(row)) << 4);
}

// Per-lane byte offsets into a swizzled tile.
//   row[ks]   : 16-byte row read, row c32, logical chunk 2*ks + g      (A/B operand over d)
//   tr[h][dt] : transposing read for d-tile dt, rows 8h + 4g + i16/4   (operand over rows)
// Add (multiple of 16 rows) * 2*D bytes for other sub-tiles; the swizzle is unchanged by that.
template <int D> struct SwzLane {
  int row[D / 16];
  int tr[2][D / 32];
  // `bias` is added to every offset (a region in front of the tiles), so that all later
  // displacements stay small enough for the 16-bit immediate of the DS instructions.
  __device__ __forceinline__ explicit SwzLane(int lane, int bias = 0) {
    const int g = lane >> 5, c32 = lane & 31, i16 = lane & 15;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) row[ks] = bias + swz_off<D>(c32, 2 * ks + g);
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt)
        tr[h][dt] = bias + swz_off<D>(8 * h + 4 * g + (i16 >> 2), dt * 4 + ((c32 >> 4) << 1) + ((i16 & 3) >> 1)) +
                    (i16 & 1) * 8;
  }
};

template <typename T>
static __device__ __forceinline__ typename Frag<T>::v8 read_tr_pair(SPARK_LDS const char* tile, int off_lo,
                                                                   int off_hi) {
  using v8 = typename Frag<T>::v8;
  using v4 = typename Frag<T>::v4;
  const v4 lo = lds_read_tr8<v4>(tile, off_lo);
  const v4 hi = lds_read_tr8<v4>(tile, off_hi);
  return join4<v8, v4>(lo, hi);
}

// Direct global->LDS copy of a swizzled ROWS x D tile: wave w of the 4 waves fills the 1 KB
// blocks w, w+4, ... of the tile; lane l writes bytes [16 l, 16 l + 16) of its block, so it
// fetches the logical chunk that the swizzle places there.  `lane_src` is that per-lane source
// offset for block `wave` (the later blocks are a multiple of 16 rows further on, where the
// swizzle repeats).  Rows past the end of the matrix arrive as zeros, and so do the chunks at
// columns >= dh: their lanes get a source offset of 2^31, which no tile offset (< 2^31, the host
// checks it) brings back inside the view.  `row_bytes` is the distance between consecutive rows
// in global memory (2*dh when the rows are contiguous).
template <int D>
static __device__ __forceinline__ uint32_t dma_lane_src(int wave, int lane, uint32_t row_bytes, int dh) {
  const int byte = wave * 1024 + lane * 16;
  const int row = byte / (2 * D), pc = (byte % (2 * D)) >> 4;
  const int chunk = pc ^ swz<D>(row);
  return chunk * 8 < dh ? (uint32_t)row * row_bytes + (uint32_t)(chunk << 4) : 0x80000000u;
}
template <int D, int ROWS>
static __device__ __forceinline__ void tile_dma(const BufView& view, int r0, SPARK_LDS char* dst,
                                                int wave, uint32_t lane_src, uint32_t row_bytes) {
  constexpr int RPG = 4 * 1024 / (2 * D);  // rows covered by one 1 KB block of each of the 4 waves
  static_assert(RPG % 16 == 0, "blocks of one wave must be 16 rows apart");
#pragma unroll
  for (int i = 0; i < ROWS * 2 * D / 4096; ++i)
    view.load16_to_lds(dst + (i * 4 + wave) * 1024, lane_src, (uint32_t)(r0 + i * RPG) * row_bytes);
}

// Write a wave's transposed accumulator (D x 32, lane = column) times `mul` as 32 rows of D
// 16-bit values: through the wave's LDS slice `ob`, then 16-byte row stores for rows < N
// and columns < dh (`row_stride` elements apart).
template <typename T, int D, int OSTR>
static __device__ __forceinline__ void store_transposed(const f32x16 (&acc)[D / 32], float mul,
                                                        SPARK_LDS char* ob, T* __restrict__ out,
                                                        int row0, int N, int lane, size_t row_stride, int dh) {
  using v4 = typename Frag<T>::v4;
  constexpr int CPR = D / 8;
  constexpr int RPP = 64 / CPR;
  const int g = lane >> 5, c32 = lane & 31;
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      v4 pk;
#pragma unroll
      for (int e = 0; e < 4; ++e) pk[e] = (T)(acc[dt][r4 * 4 + e] * mul);
      lds_write(ob, c32 * OSTR + (dt * 32 + 8 * r4 + 4 * g) * 2, pk);
    }
#pragma unroll
  for (int p = 0; p < 32 / RPP; ++p) {
    const int row = p * RPP + lane / CPR, cc = lane % CPR;
    const u32x4 v = lds_read16<u32x4>(ob, row * OSTR + cc * 16);
    if (row0 + row < N && cc * 8 < dh)
      *reinterpret_cast<u32x4*>(out + (size_t)(row0 + row) * row_stride + cc * 8) = v;
  }
}

}  // namespace spark
