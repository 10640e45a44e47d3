// Index maps of the GEMM kernels' tile movements, stated once.  The kernels compute their addresses with
// these constants and functions; axe_gemm_describe builds the layouts it reports from the same constants, and a
// test-only routine compares the reported layouts, evaluated point by point, with these functions.  Plain integer
// arithmetic, usable in host and device code.
//
// Vocabulary: an LDS tile is made of rows (one row of an operand, one K-tile wide: 64 or 128 bytes); a row is made
// of 16-byte chunks; an MFMA 16 x 16 fragment takes one row per lane l % 16 and the lane group q = l / 16 decides
// which chunks of the row the lane holds.
#pragma once

#if defined(__HIPCC__) || defined(__CUDACC__)
#define AXE_MAPS_HD __host__ __device__ constexpr
#else
#define AXE_MAPS_HD constexpr
#endif

namespace axe {
namespace maps {

constexpr int kChunkBytes = 16;
constexpr int kFrag = 16;                          // rows and columns of an MFMA fragment
constexpr int kLaneGroups = 64 / kFrag;            // lane groups of 16 lanes

// ---- LDS image: chunk c of row r sits at chunk position c ^ key(r) (the swizzle stage of the tile's layout).
//      With a key that changes every second row, 16 consecutive rows reading one logical chunk touch 16 distinct
//      16-byte bank groups, for rows of 64 bytes (4 chunks) as for rows of 128 bytes (8 chunks).
constexpr int kKeyShift = 1;
AXE_MAPS_HD int lds_key(int row, int chunks_per_row) { return (row >> kKeyShift) & (chunks_per_row - 1); }
AXE_MAPS_HD int lds_chunk_pos(int row, int chunk, int chunks_per_row) { return chunk ^ lds_key(row, chunks_per_row); }
// rows after which the key repeats: the height of the swizzle atom
AXE_MAPS_HD int lds_key_period(int chunks_per_row) { return chunks_per_row << kKeyShift; }

// ---- LDS -> VGPR: the chunk of its row that lane group q reads.
//      16-bit inputs, v_mfma_f32_16x16x32: a lane holds 8 consecutive k (one chunk); K sub-step s of the row.
AXE_MAPS_HD int operand_chunk_16bit(int s, int q) { return kLaneGroups * s + q; }
//      fp8, v_mfma_f32_16x16x128_f8f6f4: a lane holds two runs of 16 k, h = 0, 1: chunks q and q + 4 (the order in
//      which the instruction pairs the bytes of its operands; the same for A and B).
AXE_MAPS_HD int operand_chunk_fp8(int h, int q) { return q + kLaneGroups * h; }

// ---- HBM -> LDS in the 256-row kernels: one wave instruction moves kRowsPerLoad rows of 128 bytes straight into
//      1 KiB of LDS, lane l = 8 lr + lp into bytes 16 l .. 16 l + 15: LDS row lr of the piece, chunk POSITION lp,
//      so the lane fetches logical chunk lp ^ key(row).  Wave w of nw takes the pieces w, w + nw, w + 2 nw, ...
constexpr int kLargeRowBytes = 128;
constexpr int kLargeChunks = kLargeRowBytes / kChunkBytes;
constexpr int kRowsPerLoad = 64 / kLargeChunks;
AXE_MAPS_HD int piece_row(int w, int i, int lr, int nw) { return (w + nw * i) * kRowsPerLoad + lr; }

// ---- accumulator fragment with the operands swapped (B rows first): lane l holds row l % 16, columns
//      4 (l / 16) .. 4 (l / 16) + 3 in its 4 registers.
constexpr int kAccCols = 4;
// ---- paired stores: fragments j and j + 1 of a row exchange halves (v_permlane16_swap), after which lane group q
//      holds 8 consecutive columns: the first of them, counted inside the 32-column pair
AXE_MAPS_HD int pair_store_col(int q) { return (q & 1) ? kFrag + kAccCols * (q - 1) : kAccCols * q; }

static_assert(lds_key_period(kLargeChunks) == kFrag, "a fragment's 16 rows are one period of the key: the key of a fragment row depends on l % 16 alone");
static_assert(lds_key(piece_row(0, 1, 0, 4), kLargeChunks) == 0 && lds_key(piece_row(0, 1, 0, 8), kLargeChunks) == 0,
              "pieces of one wave lie whole key periods apart: a lane's key does not depend on the piece");

}  // namespace maps
}  // namespace axe
