// Plain-data descriptors handed from the host layer to the kernels by value (kernel arguments).
#pragma once
#include <stdint.h>

namespace axe {

constexpr int kMaxD = 16;
constexpr int kMaxR = 8;
constexpr int kMaxAxes = 8;
constexpr int kMaxJoint = 24;   // common refinement of two D lists can be longer than either

// XOR stage: y = x ^ (((x >> shift) & mask) << base); mask == 0 disables it.
struct Swz {
  int32_t mask, base, shift;
};

// Full layout for axe_layout_eval (all axes kept).
struct EvalDesc {
  int32_t n_d, n_r, n_axes;
  int32_t use32;               // E_D < 2^31: digit arithmetic in 32 bits
  int32_t shift[kMaxD];        // log2(ext) when ext is a power of two, else -1
  int64_t ext[kMaxD], str[kMaxD];
  int32_t axis[kMaxD];
  int64_t rext[kMaxR], rstr[kMaxR];
  int32_t raxis[kMaxR];
  int64_t off[kMaxAxes];
  int32_t swz_axis;
  Swz swz;
  int64_t E_D, E_R;
};

// Relayout plan: one loop nest shared by source and destination (their common refinement),
// enumerated fastest digit first.  Addresses in units of `unit_bytes`.
struct RelayoutPlan {
  int32_t n;                       // loop digits decoded from the thread index
  uint32_t ext[kMaxJoint];
  int32_t shift[kMaxJoint];        // log2(ext) when ext is a power of two, else -1
  int64_t ss[kMaxJoint], ds[kMaxJoint];
  int32_t U;                       // per-thread unroll digit (extent U, strides us / ud)
  int64_t us, ud;
  int64_t s_off, d_off;
  Swz s_swz, d_swz;
  int32_t n_r;                     // destination replicas
  int32_t rext[kMaxR];
  int64_t rstr[kMaxR];
  int64_t E_R;
  uint64_t threads;                // total work items = elements / (vector width * U)
  int32_t streaming;               // 1: non-temporal loads and stores (data larger than the caches)
};

// Transposing relayout: the joint loop nest has one digit that is contiguous in the source (extent
// eS, destination stride dS) and another that is contiguous in the destination (extent eD, source
// stride sD).  A workgroup moves one T x T tile of those two digits through LDS; the other digits
// (fastest first) are decoded from the workgroup index.  Addresses in elements.
struct TransposePlan {
  int32_t n;
  uint32_t ext[kMaxJoint];
  int64_t ss[kMaxJoint], ds[kMaxJoint];
  int64_t eS, eD, sD, dS;
  int64_t s_off, d_off;
  uint32_t tiles_s, tiles_d;       // tiles along the source-fast and the destination-fast digit
  uint64_t blocks;                 // tiles_s * tiles_d * product of ext[]
  int32_t streaming;               // 1: non-temporal loads and stores
  int32_t diag;                    // g > 0: tiles are walked diagonally, td = (row + ts / g) mod tiles_d; 0: row by row
  Swz s_swz, d_swz;                // swizzle stages of the two sides (mask 0: none), applied to an access's first element
  int32_t n_r;                     // destination replicas: every replica address is written
  int32_t rext[kMaxR];
  int64_t rstr[kMaxR];
  int64_t E_R;
  int32_t elementwise;             // 1: tiles of 64 x 64 moved element by element (no alignment requirement at all)
};

// Fallback when the two digit systems have no common refinement: decode each side separately.
struct GenericRelayoutPlan {
  int32_t ns, nd;
  int64_t sext[kMaxD], sstr[kMaxD];
  int64_t dext[kMaxD], dstr[kMaxD];
  int64_t s_off, d_off;
  Swz s_swz, d_swz;
  int32_t n_r;
  int32_t rext[kMaxR];
  int64_t rstr[kMaxR];
  int64_t E_R;
  int64_t total;
};

// GEMM arguments (addresses in elements of the operand's dtype).
struct GemmArgs {
  const void* A;
  const void* B;
  void* C;
  int64_t M, N, K;
  int64_t lda, ldb, ldc;           // row pitch of A (per i), of B's memory image (per j), of C (per i)
  const float* scale_a;            // (ceil(M/128), nkb) or null; bytes (E8M0 codes) when scale_e8m0
  const float* scale_b;            // (ceil(N/128), nkb) or null
  int32_t scale_e8m0;              // 1: the scale arrays hold one E8M0 byte per block (2^(code - 127))
  int32_t scale_a_rows;            // rows of A that share a scale: 128, or 1 (scale_a is then (M, nkb))
  int32_t nkb;
  int32_t out_bf16;                // 0: fp32 output, 1: 16-bit output (bf16, or binary16 when f16 is set)
  int32_t f16;                     // 1: 16-bit inputs (and a 16-bit output) are IEEE binary16 instead of bf16
  int32_t fp8;                     // grouped streaming kernel: 1 = e4m3 inputs (K-tiles of 128 elements), bf16 output
  int32_t grid_m, grid_n;          // workgroup tiles along M and N
  int32_t tile_n;                  // columns of C per workgroup tile (64, 224 or 256)
  // 256-tile bf16 kernel: operands pre-tiled along K / blocked along rows (plain matrix: kstep 128, shift 0,
  // blk_stride = tile rows x pitch)
  int32_t a_kstep, b_kstep;        // bytes between consecutive 64-wide K-tiles of one row
  int32_t a_tpb_shift, b_tpb_shift;  // log2(tiles per row block)
  int64_t a_blk_stride, b_blk_stride;  // elements between row blocks
  // grouped GEMM only: group e owns rows group_rows[e] .. group_rows[e + 1] - 1 of A and C and the matrix B + e * ldg
  const int32_t* group_rows;       // device, groups + 1 entries
  int32_t groups;
  int32_t tile_m;                  // rows of a tile of the grouped tile kernel: 128, 256, or 0 = chosen from M / groups
  int32_t compact_groups;          // streaming kernel: blockIdx.y counts non-empty groups (set by its launcher when M < groups)
  int32_t gated;                   // 1: store silu(gate) * up (B's rows interleave gate and up in runs of 16), C is N / 2 wide
  int64_t ldg;
};

// Hand-over between the two grouped GEMMs of a fused pair (the first GEMM's output is the second GEMM's A).  A row
// block of the second GEMM may be read once every column tile of the first GEMM for those rows has been stored:
// done[r] counts the stored column tiles of the row block whose first row is r (both GEMMs cut the groups into row
// blocks of the same height, so the two agree on r); done[M] counts waits that gave up.  Device memory, M + 1
// words, zero when the kernel starts.
struct PairSync {
  int32_t* done;
  int32_t need;                    // column tiles of the first GEMM per row block
  int32_t spin_limit;              // polls of done[r] before a wait gives up (the tile is then computed from what is there)
  int64_t M;
};

}  // namespace axe
