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
  __bf16* lat_o;             // [n_lat, rows, 512]
  float* lat_lse;            // [n_lat, rows]
  int Sq, H, R, Ls, ap_chunks, ap_chunk, as_chunk, max_blocks, block_size;
  int64_t rows;
  float c;                   // sm_scale * log2(e)
};

// LDS tile of 32 tokens (37888 B):
//   latent part: row r (token) at r * 1056, holding the 64 sixteen-byte chunks of its 512 latent
//     columns; chunk c sits in slot c ^ ((r >> 2) & 1).  The 32-byte row skew keeps the
//     transposing reads (4 rows x 32 B per 16 lanes) on distinct banks, the slot swizzle
//     separates rows r and r + 4 for the 16-byte reads of the score product.
//   rope part: 32 rows x 128 B behind it, chunk c of row r in slot c ^ (r & 7).
// A tile is filled by 36 wavefront-wide 1 KiB transfers: one per latent row (the swizzle is
// uniform per row) and four for the rope parts of eight rows each.  Rows past the end of the
// chunk are filled from the last valid row: their scores are masked, so they only have to be
// finite.
constexpr int AB_ROW_BYTES = 1056;
constexpr int AB_MAIN_BYTES = 32 * AB_ROW_BYTES;   // 33792
constexpr int AB_TILE_BYTES = AB_MAIN_BYTES + 32 * 128;   // 37888
constexpr int AB_DMA_PER_WAVE = 9;                 // 8 latent rows + 1 rope group per wavefront
constexpr int AB_NSLOT = 4;                        // tiles resident in LDS (3 in flight + 1 in use)
constexpr int AB_LDS_BYTES = AB_NSLOT * AB_TILE_BYTES;

// Where the 32 rows of one LDS tile come from: latent part and rope part of row i start at
// lat + i * lat_stride and rope + i * rope_stride; rows past `last` repeat row `last`.
struct RowSrc {
  const char* lat;
  const char* rope;
  int lat_stride, rope_stride, last;
};

// Per-lane constants of the tile transfers (see the tile layout above).
struct DmaLane {
  int wave, off0, off1, rope_row, rope_ch;
};

// K-th of the nine transfers with which one wavefront contributes to a tile: latent rows
// wave, wave + 4, ..., wave + 28 (K < 8), then the rope parts of rows 8*wave .. 8*wave+7 (K = 8).
// All row arithmetic is wave-uniform; the only per-lane terms are the swizzled lane offsets.
template <int K>
__device__ __attribute__((always_inline)) inline void issue_part(const RowSrc& s, char* dst,
                                                                 const DmaLane& d) {
  if constexpr (K < 8) {
    const int r = d.wave + 4 * K;          // (r >> 2) & 1 == K & 1
    const int rr = min(r, s.last);
    dma16(s.lat + (size_t)rr * s.lat_stride + ((K & 1) ? d.off1 : d.off0), dst + r * AB_ROW_BYTES);
  } else {
    const int rr = min(d.rope_row, s.last);
    dma16(s.rope + (size_t)rr * s.rope_stride + d.rope_ch, dst + AB_MAIN_BYTES + d.wave * 1024);
  }
}
__device__ __attribute__((always_inline)) inline void issue_all(const RowSrc& s, char* dst,
                                                                const DmaLane& d) {
  static_for<AB_DMA_PER_WAVE>([&](auto k) { issue_part<decltype(k)::value>(s, dst, d); });
}

int mfma_absorb64_attention(const Plan& p, const DecodeArgs& d, const AbsorbArgs& a);

}  // namespace tmla
