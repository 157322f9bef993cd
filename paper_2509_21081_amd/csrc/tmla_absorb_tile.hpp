// Pieces shared by the absorb-formulation attention kernels for 32 or more query rows per
// request (paper Algorithm 1 step 6): kernel arguments, the LDS tile of 32 latent cache rows and
// the global -> LDS transfers that fill it.
#pragma once
#include <type_traits>
#include <utility>

#include "tmla_common.hpp"
#include "tmla_lds_asm.hpp"
#include "tmla_mfma.hpp"

namespace tmla {

struct AbsorbArgs {
  const __bf16* qabs;        // [rows, 576]
  const __bf16* pc;          // prefix latent [Ls, 512]  (absorb_only)
  const __bf16* pr;          // prefix rope   [Ls, 64]
  const __bf16* pool;        // [num_blocks, block_size, 576]
  const int32_t* block_table;
  const int32_t* lens;
  const int32_t* order;      // workgroup's request slot -> request, or nullptr (identity)
  __bf16* lat_o;             // [n_lat, rows, 512]
  float* lat_lse;            // [n_lat, rows]
  int Sq, H, R, Ls, ap_chunks, ap_chunk, as_chunk, max_blocks, block_size;
  int64_t rows;
  float c;                   // sm_scale * log2(e)
};

// LDS tile of 32 tokens (38912 B).  The LDS has 64 four-byte banks; a 16-byte read is served 16
// consecutive lanes at a time, an 8-byte (transposing) read 32 lanes at a time, and a group is
// conflict-free when its lanes cover all 64 banks once.
//   latent part: row r (token) at r * 1088, holding the 64 sixteen-byte chunks of its 512 latent
//     columns; chunk c sits in slot c ^ ((r >> 2) & 3).  The row stride is 16 banks mod 64, so
//     the transposing reads (4 rows x 64 B per 32 lanes) cover the banks exactly; the slot
//     swizzle separates rows r, r + 4, r + 8, r + 12 for the 16-byte reads of the score product
//     (16 rows, one chunk each).  The 64 bytes behind a row's chunks are never written by a
//     transfer (the 64-row kernel keeps its row maxima there).
//   rope part: 32 rows x 128 B behind it, chunk c of row r in slot c ^ ((r >> 1) & 7): rows of
//     equal parity share 32 banks and are separated by the swizzle.
// A tile is filled by 36 wavefront-wide 1 KiB transfers: one per latent row (the swizzle is
// uniform per row) and four for the rope parts of eight rows each.  Rows past the end of the
// chunk are filled from the last valid row: their scores are masked, so they only have to be
// finite.
constexpr int AB_ROW_BYTES = 1088;
constexpr int AB_MAIN_BYTES = 32 * AB_ROW_BYTES;   // 34816
constexpr int AB_TILE_BYTES = AB_MAIN_BYTES + 32 * 128;   // 38912
constexpr int AB_DMA_PER_WAVE = 9;                 // 8 latent rows + 1 rope group per wavefront
constexpr int AB_NSLOT = 4;                        // tiles resident in LDS (3 in flight + 1 in use)
constexpr int AB_LDS_BYTES = AB_NSLOT * AB_TILE_BYTES;   // 155648

// Per-lane byte offsets into a tile for the three read patterns (lane = n + 32 g):
//   score product, latent k-step ks < 32: row n, chunk 2 ks + g -> s_off[ks & 1] + 64 (ks >> 1)
//   score product, rope k-step 32 + k   : row n, chunk 2 k + g  -> r_off[k]
//   output product (transposing 8-byte reads; 16-lane group j = lane / 16, r = lane % 16):
//     token row 4 g + r / 4 (v_lo) or that + 8 (v_hi), latent columns 16 (j % 2) + 4 (r % 4) ..+3
//     of a 32-column block; the caller adds 16 rows per further k-step and 64 B per block.
struct TileLane {
  uint32_t s_off[2], r_off[4], v_lo, v_hi;
};
__device__ inline TileLane tile_lane(int lane) {
  const int n = lane & 31, g = lane >> 5, sw = (n >> 2) & 3;
  TileLane t;
#pragma unroll
  for (int par = 0; par < 2; par++) t.s_off[par] = n * AB_ROW_BYTES + (((2 * par + g) ^ sw) << 4);
#pragma unroll
  for (int k = 0; k < 4; k++)
    t.r_off[k] = AB_MAIN_BYTES + n * 128 + (((2 * k + g) ^ ((n >> 1) & 7)) << 4);
  const int j16 = lane >> 4, r16 = lane & 15;
  const int chunk = 2 * (j16 & 1) + ((r16 & 3) >> 1);
  const uint32_t row = (4 * g + (r16 >> 2)) * AB_ROW_BYTES + 8 * (r16 & 1);
  // rows 16 kk + 4 g + 0..3 have swizzle g, rows 8 further down g ^ 2
  t.v_lo = row + ((chunk ^ g) << 4);
  t.v_hi = row + 8 * AB_ROW_BYTES + ((chunk ^ g ^ 2) << 4);
  return t;
}
// fragment of latent k-step KS (rows = the tile's 32 tokens) for the score product
template <int KS>
__device__ inline bf16x8 tile_score_frag(uint32_t tile, const TileLane& t) {
  return lds_read_b128<64 * (KS >> 1)>(tile + t.s_off[KS & 1]);
}

// Where the 32 rows of one LDS tile come from: latent part and rope part of row i start at
// lat + i * lat_stride and rope + i * rope_stride; rows past `last` repeat row `last`.
struct RowSrc {
  const char* lat;
  const char* rope;
  int lat_stride, rope_stride, last;
  bool stream;   // rows nobody else reads (a request's own suffix): non-temporal transfers
};

// Per-lane constants of the tile transfers (see the tile layout above).
struct DmaLane {
  int wave, off[4], rope_row, rope_ch;
};
__device__ inline DmaLane dma_lane(int wave, int lane) {
  DmaLane d;
  d.wave = wave;
#pragma unroll
  for (int sw = 0; sw < 4; sw++) d.off[sw] = (lane ^ sw) << 4;
  d.rope_row = 8 * wave + (lane >> 3);
  d.rope_ch = ((lane & 7) ^ ((d.rope_row >> 1) & 7)) << 4;
  return d;
}

// K-th of the nine transfers with which one wavefront contributes to a tile: latent rows
// wave, wave + 4, ..., wave + 28 (K < 8), then the rope parts of rows 8*wave .. 8*wave+7 (K = 8).
// All row arithmetic is wave-uniform; the only per-lane terms are the swizzled lane offsets.
template <int K>
__device__ __attribute__((always_inline)) inline void issue_part(const RowSrc& s, char* dst,
                                                                 const DmaLane& d) {
  if constexpr (K < 8) {
    const int r = d.wave + 4 * K;          // (r >> 2) & 3 == K & 3
    const int rr = min(r, s.last);
    if (s.stream) dma16_stream(s.lat + (size_t)rr * s.lat_stride + d.off[K & 3], dst + r * AB_ROW_BYTES);
    else dma16(s.lat + (size_t)rr * s.lat_stride + d.off[K & 3], dst + r * AB_ROW_BYTES);
  } else {
    const int rr = min(d.rope_row, s.last);
    if (s.stream) dma16_stream(s.rope + (size_t)rr * s.rope_stride + d.rope_ch, dst + AB_MAIN_BYTES + d.wave * 1024);
    else dma16(s.rope + (size_t)rr * s.rope_stride + d.rope_ch, dst + AB_MAIN_BYTES + d.wave * 1024);
  }
}
__device__ __attribute__((always_inline)) inline void issue_all(const RowSrc& s, char* dst,
                                                                const DmaLane& d) {
  static_for<AB_DMA_PER_WAVE>([&](auto k) { issue_part<decltype(k)::value>(s, dst, d); });
}

int mfma_absorb64_attention(const Plan& p, const DecodeArgs& d, const AbsorbArgs& a);
int mfma_absorb128_attention(const Plan& p, const DecodeArgs& d, const AbsorbArgs& a);

}  // namespace tmla
