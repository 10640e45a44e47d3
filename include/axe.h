/* axe.h -- C ABI of the MI355X (gfx950) Axe-layout hot path.
 *
 * Three operations, each driven by Axe layouts (Sec. 2 of the paper: a layout is a shard list
 * D of iters (extent, stride, named axis), a replica multiset R and a per-axis offset O; the
 * induced map is f_L(x) = { f_D(x) + f_R(r) + O }):
 *
 *   axe_layout_eval   evaluate the induced map on the GPU                     (Sec. 2.3, Def. 2.3)
 *   axe_relayout      copy one logical tensor from one layout to another      (Sec. 3.2, `copy` operator)
 *   axe_gemm          layout-driven tiled dense GEMM, bf16 / block-scaled fp8 (Sec. 3.2 `gemm` operator,
 *                                                                              Sec. 4.1 workloads)
 *
 * Conventions common to all entry points
 *   - Pointers named d_* are DEVICE pointers (HIP global memory on the current device); every
 *     other pointer is a HOST pointer.  The caller owns all of them; descriptors are read during
 *     the call and never retained.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued
 *     asynchronously on it; the call returns without synchronising.
 *   - Return value: AXE_OK (0) or a negative error code; nothing is launched when an error is
 *     returned.  No call aborts or throws.  axe_strerror() names a code, axe_last_error() gives
 *     the detailed message of the calling thread's last failure.
 *   - The library keeps no global mutable state apart from that thread-local message, and
 *     allocates no device memory.
 *   - One GPU holds the whole tensor: an axis other than the memory axis may appear only with
 *     total extent 1 (e.g. the extent-1 `gpuid` iter and `gpuid` offset of one shard of a
 *     sharded tensor, Sec. 2.2); such iters are removed by canonicalisation rule D0 (App. A)
 *     and offsets on such axes do not enter addresses.
 */
#ifndef AXE_H
#define AXE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AXE_MAX_D     16   /* sharded iters per layout                 */
#define AXE_MAX_R      8   /* replica iters per layout                 */
#define AXE_MAX_AXES   8   /* named axes per layout                    */
#define AXE_MAX_RANK   8   /* logical shape rank                       */

enum {
  AXE_OK           =  0,
  AXE_EINVAL       = -1,  /* violates Def. 2.1 / 2.2: extent <= 0, stride == 0, n_d < 1, axis out of range,
                             bad swizzle, NULL where a pointer is required, too many iters            */
  AXE_ESHAPE       = -2,  /* shape not admitted (prod(shape) != E_D, Sec. 2.3) or shapes inconsistent  */
  AXE_EALIAS       = -3,  /* a destination is not injective on the memory axis (two logical elements
                             share an address), or a non-memory axis has extent > 1 on one GPU        */
  AXE_ERANGE       = -4,  /* an address falls outside the declared buffer, or arithmetic overflows    */
  AXE_EUNSUPPORTED = -5,  /* valid layouts outside the kernel families of this library               */
  AXE_EHIP         = -6,  /* HIP runtime failure (launch error)                                       */
  AXE_ENOFORM      = -7,  /* a layout operator's sufficient conditions do not hold (the paper's FAILURE
                             outcome of grouping, tile-of and slice): valid inputs, no answer of the
                             required form                                                             */
  AXE_ETIMEOUT     = -8   /* a bounded wait inside a kernel gave up (axe_gemm_grouped_pair_status)        */
};

/* Def. 2.1: f_I(x) = (x * stride) @ axis;  extent > 0, stride != 0, 0 <= axis < n_axes. */
typedef struct {
  int64_t extent;
  int64_t stride;
  int32_t axis;
} axe_iter_t;

/* Def. 2.2 plus the swizzle stage.
 * D is ordered (first iter = slowest digit of the lexicographic unflattening); R is a multiset,
 * evaluated in the order written (last iter fastest).  offset has n_axes entries or is NULL (all 0).
 * Swizzle (Sec. 3.4 models the hardware swizzle as a separate innermost layout; here it is one
 * stage applied to the coordinate on axis swz_axis after D + R + O):
 *     y = x ^ (((x >> swz_shift) & (2^swz_bits - 1)) << swz_base),  swz_base + swz_bits <= swz_shift,
 * swz_axis = -1 disables it.  The coordinate must be non-negative where a swizzle applies. */
typedef struct {
  int32_t           n_axes;      /* 1..AXE_MAX_AXES                                        */
  const char* const* axis_names; /* n_axes labels for messages, or NULL                    */
  int32_t           n_d;         /* 1..AXE_MAX_D                                           */
  const axe_iter_t* d;
  int32_t           n_r;         /* 0..AXE_MAX_R                                           */
  const axe_iter_t* r;           /* may be NULL when n_r == 0                              */
  const int64_t*    offset;
  int32_t           swz_axis, swz_bits, swz_base, swz_shift;
} axe_layout_t;

/* ---------------------------------------------------------------------------------------------
 * axe_layout_eval -- the induced map f_{L<S>} of Def. 2.3 / "Shape admission" (Sec. 2.3).
 *
 *   L, rank, shape : layout and a shape it admits (prod(shape) == E_D), rank 1..AXE_MAX_RANK.
 *   n              : number of logical indices to evaluate.
 *   d_flat_idx     : DEVICE, n row-major flattened logical indices in [0, E_D); NULL = 0..n-1
 *                    (then n <= E_D is required).  Indices outside the range produce
 *                    INT64_MIN in every output slot of that index (no out-of-bounds access).
 *   d_out          : DEVICE, n * E_R * n_axes int64, laid out [index][replica][axis]; replica t
 *                    enumerates R lexicographically in the order written (last iter fastest).
 * Bit-exact integer arithmetic (int64, two's complement). */
int axe_layout_eval(const axe_layout_t* L, int32_t rank, const int64_t* shape,
                    int64_t n, const int64_t* d_flat_idx, int64_t* d_out, void* stream);

/* ---------------------------------------------------------------------------------------------
 * axe_relayout -- dst[f_dst(x)] = src[f_src(x)] for every logical index x of `shape`
 * (the `copy` operator between two layouts of the same logical tensor, Sec. 3.2; blocked
 * destinations are tile products, Sec. 3.3; swizzled ones use the stage above).
 *
 *   src, dst     : layouts admitting `shape`.  Addresses are the coordinates on axis `mem_axis`
 *                  (same index in both layouts), in units of elements.
 *   elem_bytes   : 1, 2, 4, 8 or 16.
 *   d_src, d_dst : DEVICE buffers of src_elems / dst_elems elements, aligned to elem_bytes;
 *                  they must not overlap.
 * Semantics of replication: every replica address of dst is written; src is read at its first
 * replica (all replica digits 0).  Words of dst no logical index maps to are left untouched.
 * Data are moved as raw bits (no float interpretation).
 * Errors: AXE_ESHAPE, AXE_EALIAS (dst not provably injective, replicas included: two (logical
 * element, replica) pairs could write one address -- the test is the sufficient one: the shard and
 * replica iters on the memory axis, sorted by |stride|, must each step over the span of all smaller
 * ones), AXE_ERANGE (some address outside [0, *_elems)), AXE_EINVAL. */
int axe_relayout(const axe_layout_t* src, const axe_layout_t* dst, int32_t rank, const int64_t* shape,
                 int32_t elem_bytes, int32_t mem_axis,
                 const void* d_src, int64_t src_elems, void* d_dst, int64_t dst_elems, void* stream);

/* ---------------------------------------------------------------------------------------------
 * axe_gemm -- C[i][j] = sum_k A[i][k] * B[k][j], fp32 accumulation on the MFMA units
 * (dense GEMM, Sec. 4.1; tiles are moved HBM -> LDS -> registers -> MFMA -> HBM following the
 * layouts reported by axe_gemm_describe).
 *
 *   A : logical shape (M, K);  B : logical shape (K, N);  C : logical shape (M, N); each with its
 *       layout on the memory axis `mem_axis`, addresses in elements of the tensor's dtype.
 *   in_dtype  : AXE_BF16 (2 bytes), AXE_F16 (IEEE binary16; the fused MoE layer of Sec. 4.1 is an FP16
 *               layer) or AXE_FP8_E4M3 (1 byte, OCP e4m3: max 448, no inf).
 *   out_dtype : AXE_F32, or the 16-bit type that goes with the inputs -- AXE_BF16 for bf16 and fp8 inputs,
 *               AXE_F16 for fp16 inputs (round to nearest even from the fp32 accumulator).
 *   d_scale_a, d_scale_b : both NULL, or DEVICE arrays of scale_dtype, row-major (ceil(M/sb), ceil(K/sb))
 *       and (ceil(N/sb), ceil(K/sb)) with sb = scale_block (must be 128):
 *       C[i][j] = sum_kb sA[i/sb][kb] * sB[j/sb][kb] * sum_{k in block kb} A[i][k] B[k][j]
 *       (block-wise scaled GEMM, Sec. 4.1).  Only with AXE_FP8_E4M3.  With scale_a_rows = 1 the scales
 *       of A are one per row and k block, d_scale_a row-major (M, ceil(K/sb)), sA[i][kb] in the formula.
 *   scale_dtype : AXE_SCALE_F32 (0; fp32 scales, folded on the vector ALU) or AXE_SCALE_E8M0 (one byte
 *       per block, value 2^(code - 127), codes 1..254; the "FP8 (e8m0) block-wise scaling" of Sec. 4.1,
 *       applied by the matrix cores' own scale path).  E8M0 arrays must be 4-byte aligned.
 *   a_elems, b_elems, c_elems : sizes of the device buffers in elements (range check).
 * Supported family (else AXE_EUNSUPPORTED): after canonicalisation A and B have unit stride
 * along k and C has unit stride along j (A row-major, B column-major, C row-major, any leading
 * dimensions that are multiples of 16 bytes, any offsets that keep 16-byte alignment); K a
 * multiple of 16 bytes' worth of elements.  For the 256 x 256 tile with 16-bit inputs, A and B may also be
 * stored in blocks (Sec. 3.3, a tile product): along k the grouped form (K/64, s)(64, 1), along the other
 * dimension (R/rb, S)(rb, pitch) with rb = 256 x 2^n.  d_C must not overlap d_A or d_B. */
enum { AXE_BF16 = 1, AXE_FP8_E4M3 = 2, AXE_F32 = 3, AXE_F16 = 4 };

typedef struct {
  int64_t      M, N, K;
  int32_t      in_dtype, out_dtype;
  axe_layout_t A, B, C;
  int32_t      mem_axis;
  int64_t      a_elems, b_elems, c_elems;
  const void*  d_scale_a;   /* fp32 or E8M0 (uint8) arrays, see scale_dtype */
  const void*  d_scale_b;
  int32_t      scale_block;
  int32_t      tile_hint;   /* 0 = library default; AXE_TILE_* forces a kernel (AXE_EUNSUPPORTED if
                               the shape does not fit it)                                         */
  int32_t      scale_dtype; /* AXE_SCALE_F32 or AXE_SCALE_E8M0                                    */
  int32_t      scale_a_rows; /* rows of A that share a scale: 0 or 128 = square blocks; 1 = one scale per
                                row and 128-wide k block (activations; d_scale_a is then (M, ceil(K/128)));
                                B keeps 128 x 128 blocks.  Served by the 64 x 64 kernel, and with E8M0
                                codes, K a multiple of 1024 and M, N multiples of 256 by the 256 x 256
                                kernel on the matrix cores' scale path.                                */
} axe_gemm_desc_t;

enum { AXE_SCALE_F32 = 0, AXE_SCALE_E8M0 = 1 };

enum { AXE_TILE_AUTO = 0, AXE_TILE_64x64x32 = 1, AXE_TILE_256x256x64 = 2, AXE_TILE_256x224x64 = 3 };

int axe_gemm(const axe_gemm_desc_t* g, const void* d_A, const void* d_B, void* d_C, void* stream);

/* The kernel axe_gemm would launch for `g` (host only, device pointers not needed):
 * returns AXE_TILE_64x64x32, AXE_TILE_256x256x64 or AXE_TILE_256x224x64 (bf16 only: 224 columns of C
 * per workgroup, chosen when N is a multiple of 224 and the tile count then fills the compute units
 * better, e.g. N = 3584 with M = 4096), or the error axe_gemm would return.
 * Shapes: the 64 x 64 tile takes any M and N.  The 256 x 256 tile needs K a multiple of 64 (fp8: 128); with fp8
 * inputs a 16-bit output and M and N multiples of 256; with 16-bit inputs a 16-bit or an fp32 output, any M and
 * any N that is a multiple of 8 (fp32 output: of 4) -- edges that do not fill a tile are cut off by the buffer
 * bounds (plain operands only).  Left to itself the library takes the large tile once
 * M x N reaches 5 x 2^20 elements (fp8: 2^20); below that the 64 x 64 tiles are faster (a single large tile
 * takes as long as several rounds of small ones). */
int axe_gemm_tile(const axe_gemm_desc_t* g);

/* ---------------------------------------------------------------------------------------------
 * axe_gemm_grouped -- the grouped GEMM of a mixture-of-experts layer (Sec. 4.1, "fused MoE layer": its
 * two group GEMMs): the rows of A and C are sorted by group (expert), group e owns the rows
 * group_rows[e] .. group_rows[e+1]-1 and has its own right-hand side,
 *       C[r, j] = sum_k A[r, k] * B[e, k, j]      for group_rows[e] <= r < group_rows[e+1].
 * Rows that belong to no group (below group_rows[0], from group_rows[G] on) are not written.
 *
 *   M, N, K : logical sizes; M = rows of A and C, all groups together (any positive value).
 *   G       : number of groups, 1..4096.
 *   A : (M, K), B : (G, K, N), C : (M, N)  Axe layouts on `mem_axis`, in elements.
 *   d_A, d_B, d_C  : DEVICE buffers of a_elems / b_elems / c_elems elements, 16-byte aligned;
 *                    d_C must not overlap d_A or d_B.
 *   d_group_rows   : DEVICE, G + 1 int32, non-decreasing, within [0, M].  The host never reads them
 *                    (a router writes them on the device): the kernel clamps each entry to [0, M], so
 *                    no access leaves the buffers whatever they hold; entries that decrease give
 *                    unspecified values in C.
 * Supported family (else AXE_EUNSUPPORTED): bf16 inputs and output, fp16 inputs and output, or fp8 inputs with bf16
 * output (see the scale fields below); A and C row-major, each B[e]
 * column-major (unit stride along k) with one pitch for all e and a constant stride between groups
 * (the grouped form of B by (G, K, N) has one iter per block); leading dimensions, offsets and the group
 * stride multiples of 16 bytes; N a multiple of 256, K a multiple of 64.
 * One launch, work found on the device from d_group_rows; nothing is allocated and no scratch memory
 * is used.  G = 1 with d_group_rows = {0, M} is a dense GEMM; with few rows (M <= 64) that is the way to
 * the weight-streaming kernel (8192 x 8192 bf16 weights, M = 16: 33 us, against 125 us of axe_gemm's
 * 64 x 64 kernel). */
typedef struct {
  int64_t      M, N, K;
  int32_t      G;
  int32_t      in_dtype, out_dtype;      /* both AXE_BF16, both AXE_F16, or AXE_FP8_E4M3 with AXE_BF16 */
  axe_layout_t A, B, C;
  int32_t      mem_axis;
  int64_t      a_elems, b_elems, c_elems;
  int32_t      epilogue;                 /* AXE_EPI_NONE or AXE_EPI_SWIGLU */
  int32_t      kernel_hint;              /* AXE_GROUPED_AUTO, or one of the two kernels below */
  const void*  d_scale_a;                /* fp8 only: both NULL, or DEVICE block scales (see below) */
  const void*  d_scale_b;
  int32_t      scale_dtype;              /* AXE_SCALE_F32 or AXE_SCALE_E8M0 */
} axe_gemm_grouped_desc_t;

/* fp8 (in_dtype AXE_FP8_E4M3, out_dtype AXE_BF16): the block-scaled grouped GEMM of an fp8 MoE layer,
 *       C[r, j] = sum_kb sA[r][kb] * sB[e][j / 128][kb] * sum_{k in block kb} A[r, k] B[e, k, j],   blocks of 128 along k,
 * d_scale_a row-major (M, ceil(K/128)): one scale per row of A and k block (activations), d_scale_b row-major
 * (G, N/128, ceil(K/128)): one per 128 x 128 block of each B[e]; fp32, or E8M0 codes (one byte, 2^(code - 127);
 * such arrays are read in aligned 4-byte words: 4-byte aligned, allocation padded to a multiple of 4 bytes).
 * Both NULL: unscaled.  K a multiple of 128; B[e] column-major (plain, or gate/up interleaved for the gated
 * epilogue).  Two kernels: the streaming kernel (any scales; groups of more than 64 rows take several passes over
 * their weights), and, with E8M0 scales or none, the tile kernel on the matrix cores' scale path (tiles of 256
 * or 128 rows: kernel_hint AXE_GROUPED_TILES, _256 or _128; gated: N / 2 a multiple of 128; AUTO takes it
 * from 9 rows per group on average, 16 when K <= 1024, with 128-row tiles up to 384 rows per group).  A hint
 * that asks for tiles with fp32 scales is AXE_EUNSUPPORTED. */

/* Two kernels serve the same family.  AXE_GROUPED_TILES: 256 x 256 tiles of the chained GEMM pipeline, for
 * groups of hundreds of rows (of 128 x 256 unless groups average more than 384 rows: a K-step then takes half
 * the matrix-core time and the weights stream past faster).  AXE_GROUPED_STREAM: one workgroup per (group, 128 rows of B), the group's
 * rows (16, 32 or 64 at a time) held in registers while its weights stream by once -- for the few rows per group of
 * an MoE layer at decode batch sizes, where the time is that of reading the weights.  AUTO takes the
 * streaming kernel when M <= 13 G, or M <= 19 G when K <= 1024 (the host knows M, not the group sizes; measured
 * crossovers on the two GEMMs of the benchmark's MoE layer).  In a pair the second GEMM follows the first. */
enum { AXE_GROUPED_AUTO = 0, AXE_GROUPED_TILES = 1, AXE_GROUPED_STREAM = 2,
       /* the tile kernel with tiles of 256 or 128 rows (AXE_GROUPED_TILES takes 128 while M <= 384 G) */
       AXE_GROUPED_TILES_256 = 3, AXE_GROUPED_TILES_128 = 4 };

/* AXE_EPI_SWIGLU: the gated activation between the two group GEMMs, fused into the first.  The logical
 * columns [0, N/2) of every B[e] are the gate projection, [N/2, N) the up projection, C is (M, N/2):
 *       C[r, c] = silu(P[r, c]) * P[r, c + N/2],   P = A B[e] in fp32,   silu(x) = x / (1 + exp(-x)).
 * Supported family: as above, and gate and up columns interleaved in memory in runs of 16 rows of the
 * group's image (logical column h N/2 + 16 f + i in row 32 f + 16 h + i): along n the grouped form of B is
 * (2, 16 p)(N/32, 32 p)(16, p), or (2, 16 p)(N/256, S)(8, 32 p)(16, p) for 256-row blocks; axe_relayout
 * produces either from the plain matrix. */
enum { AXE_EPI_NONE = 0, AXE_EPI_SWIGLU = 1 };

int axe_gemm_grouped(const axe_gemm_grouped_desc_t* g, const void* d_A, const void* d_B, void* d_C,
                     const int32_t* d_group_rows, void* stream);
/* The checks of axe_gemm_grouped without a launch (host only): AXE_OK or the error it would return. */
int axe_gemm_grouped_check(const axe_gemm_grouped_desc_t* g);

/* ---------------------------------------------------------------------------------------------
 * axe_gemm_grouped_pair -- the expert computation of an MoE layer as ONE launch (Sec. 4.1, "fused MoE layer": the
 * two group GEMMs overlap through a tile-level dependency instead of a kernel boundary):
 *       H = epilogue1(A B1[e])   (problem g1, gated activation),      C = H B2[e]   (problem g2, no epilogue),
 * where g2's A is g1's C: same M, G, element type and count, same layout, K2 = columns of H.  The row blocks of
 * the second GEMM start as soon as the column tiles of the first GEMM for those rows are stored; the workgroups that
 * run out of tiles of the first GEMM go on with the second.  d_H is an output like d_C (the intermediate activations,
 * rounded to the 16-bit type exactly as axe_gemm_grouped stores them: the result equals two axe_gemm_grouped calls).
 *
 *   d_A, d_B1, d_B2, d_group_rows : DEVICE inputs, as for axe_gemm_grouped (one d_group_rows for both problems).
 *   d_H, d_C : DEVICE outputs, disjoint from the inputs and from each other.
 *   d_sync, sync_elems : DEVICE workspace of at least M + 1 int32 words (4-byte aligned), owned by the caller,
 *       overwritten by every call (cleared on the stream by a small kernel, so the call may be captured into a
 *       graph); calls that share one d_sync must not overlap in time.  NULL: the two problems run one after the
 *       other on the stream, as they also do when they cannot share a launch -- 16-bit tile kernels of the same
 *       tile height only, both K multiples of 128 and at least 256, first problem gated, H's rows starting on
 *       128-byte boundaries (pitch and buffer), and few enough tiles that one workgroup per compute unit holds
 *       them (64 per workgroup and problem).
 *   Every wait inside the kernel is bounded (a number of polls, AXE_GROUPED_PAIR_POLLS, default 2^20, each a few
 *   microseconds): a wait that gives up is counted in d_sync[M] and the tile is computed from what is there.
 *   axe_gemm_grouped_pair_status(d_sync, M, stream) synchronises the stream and returns AXE_ETIMEOUT if any wait of
 *   the last call gave up (rows of C are then invalid), else AXE_OK (d_sync NULL: see axe_gemm_grouped_pair_static).  With all workgroups resident (the launch is
 *   sized to the compute units of the device) no wait can fail to end: tiles of the first GEMM wait for nothing and
 *   every workgroup works through its share of them before it waits.  Other work that keeps compute units from this
 *   launch (kernels of other streams or processes) only delays the waits, unless it does so for longer than the poll
 *   limit allows (seconds): then waits give up and the status call says so.
 *   axe_gemm_grouped_pair_fused(g1, g2): 1 if the pair would share a launch (given a workspace), 0 if not, or the
 *   error axe_gemm_grouped_pair would return (host only).
 * Errors: those of axe_gemm_grouped for either problem; AXE_EINVAL when g2's A is not g1's C, when H or C overlaps
 * the other or an input of either problem, or when the workspace is too small or overlaps an operand. */
int axe_gemm_grouped_pair(const axe_gemm_grouped_desc_t* g1, const axe_gemm_grouped_desc_t* g2, const void* d_A,
                          const void* d_B1, void* d_H, const void* d_B2, void* d_C, const int32_t* d_group_rows,
                          int32_t* d_sync, int64_t sync_elems, void* stream);
int axe_gemm_grouped_pair_fused(const axe_gemm_grouped_desc_t* g1, const axe_gemm_grouped_desc_t* g2);
int axe_gemm_grouped_pair_status(const int32_t* d_sync, int64_t M, void* stream);

/* axe_gemm_grouped_pair_static -- axe_gemm_grouped_pair for callers that cannot allocate device memory or hand a
 * workspace through: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * counters live in an array of the library's own (a __device__ array of 2^20 + 1 words, 4 MiB of every device the
 * library runs on, held until the process ends); the call allocates nothing and frees nothing.  Same arguments
 * and results as axe_gemm_grouped_pair without d_sync / sync_elems; M above 2^20 rows is AXE_EUNSUPPORTED.  All
 * calls on one device share the array: calls that overlap in time on one device (different streams) race on it
 * -- give such callers workspaces of their own through axe_gemm_grouped_pair.  The array keeps the last call's
 * counts; every call clears the M + 1 words it uses, on the stream, with a small kernel.  The first call on a device
 * asks the runtime for the array's address: make that call outside graph capture (the warm-up run a capture needs
 * anyway does it).
 * axe_gemm_grouped_pair_status(NULL, M, stream) reads the status word of the last such call on the current device. */
int axe_gemm_grouped_pair_static(const axe_gemm_grouped_desc_t* g1, const axe_gemm_grouped_desc_t* g2, const void* d_A,
                                 const void* d_B1, void* d_H, const void* d_B2, void* d_C, const int32_t* d_group_rows,
                                 void* stream);

/* ---------------------------------------------------------------------------------------------
 * axe_gemm_describe -- the Axe layouts of every tile movement of the kernel axe_gemm would
 * launch for `g` (Sec. 3.1 / Fig. 3: tensors in shared memory and registers carry layouts; tile
 * composes register tile (x) lane (x) wave (x) workgroup, Sec. 3.3).  Host only, no device work.
 *
 *   which : AXE_DESC_*.
 *   out   : receives the layout; its d / r / offset / axis_names pointers point into `arena`.
 *   shape, rank : receive the logical shape the layout admits (up to AXE_MAX_RANK entries).
 *   arena, arena_bytes : caller-provided HOST scratch (2 KiB is enough).
 * Axis names used: "m" (HBM element address), "lds" (LDS element address), "wg", "wave", "lane",
 * "reg" (index of the element inside the lane's fragment / accumulator / per-thread loop).
 * In the thread maps of operands that are loaded straight into LDS by the 256 x 256 kernels the
 * swizzle key spans the wave id; those maps are stated on the thread id, folded into the "lane"
 * axis as lane + 64 * wave (extent 64 * waves), with "wave" unused.
 * AXE_EUNSUPPORTED is never returned for a descriptor axe_gemm accepts. */
enum {
  AXE_DESC_A_G2L_THREADS = 0, /* (BM, BK) tile of A  -> wave, lane, reg : who fetches which element  */
  AXE_DESC_B_G2L_THREADS = 1,
  AXE_DESC_A_LDS         = 2, /* (BM, BK) tile of A  -> lds (with swizzle) for one stage             */
  AXE_DESC_B_LDS         = 3,
  AXE_DESC_A_OPERAND     = 4, /* (BM, BK) tile of A  -> wave(s, replicated), lane, reg (MFMA operand)*/
  AXE_DESC_B_OPERAND     = 5,
  AXE_DESC_ACC           = 6, /* (M, N) of the whole problem -> wg, wave, lane, reg (accumulators)   */
  AXE_DESC_C_STORE       = 7  /* (BM, BN) tile of C  -> wave, lane, reg : who stores which element   */
};
int axe_gemm_describe(const axe_gemm_desc_t* g, int32_t which, axe_layout_t* out,
                      int64_t* shape, int32_t* rank, void* arena, size_t arena_bytes);

/* The same for axe_gemm_grouped (Sec. 4.1, fused MoE layer; host only).  The grouped tile kernels are the dense
 * 256-wide 16-bit kernel at a tile height of 256 or 128 rows and report its layouts at that height; AXE_DESC_ACC is
 * the accumulator layout of one tile (where a tile lies in the problem depends on the group sizes, which only the
 * device knows).  AXE_EUNSUPPORTED: the streaming kernel (no LDS stage; its register maps are stated in its source),
 * and AXE_DESC_C_STORE with the gated epilogue (a stored element comes from two accumulators).
 * axe_gemm_grouped_kernel returns the kernel axe_gemm_grouped would launch: AXE_GROUPED_STREAM,
 * AXE_GROUPED_TILES_256 or AXE_GROUPED_TILES_128, or the error axe_gemm_grouped would return. */
int axe_gemm_grouped_kernel(const axe_gemm_grouped_desc_t* g);
int axe_gemm_grouped_describe(const axe_gemm_grouped_desc_t* g, int32_t which, axe_layout_t* out,
                              int64_t* shape, int32_t* rank, void* arena, size_t arena_bytes);

/* ---------------------------------------------------------------------------------------------
 * Layout operators (Sec. 3.3; Apps. A - F).  Host only: pure integer bookkeeping on (D, R, O),
 * nothing is launched.  Results are written through `out`, whose d / r / offset pointers point
 * into the caller's HOST `arena` (1 KiB is always enough); out->axis_names is the first operand's.
 * Operands of one call must share one axis list (equal n_axes).  A result with more than
 * AXE_MAX_D / AXE_MAX_R iters is AXE_ERANGE.
 *
 *   axe_layout_span          span[a] = 1 + sum |stride| (extent - 1) over the D and R iters on axis a
 *                            (Sec. 2.3; O does not enter); span has n_axes entries.
 *   axe_layout_canonicalize  App. A: D0 (drop unit iters), D1 (fuse a chain (e1, e2 s2)(e2, s2) on one
 *                            axis) on D; C0 (drop unit iters), C1 (strides positive, the reach goes
 *                            into O), C2 (absorb (e2, q s) into (e1, s) when 1 <= q <= e1) on (R, O).
 *                            R comes out sorted by (axis, stride, extent).  A swizzle stage is kept.
 *   axe_layout_gap_condition 1 if the sign-normalised replicas satisfy the gap condition (per axis,
 *                            strides increasing, each above extent x stride of the one before), under
 *                            which the canonical form is unique; 0 if not; negative on error.
 *   axe_layout_equal         1 if the canonical forms (and swizzle stages) coincide, else 0; a 0 is
 *                            conclusive when both operands satisfy the gap condition.
 *   axe_layout_group         Alg. 1: the same map with D cut into `rank` consecutive blocks whose
 *                            extent products are shape[i] (iters split by gcd where they straddle a
 *                            boundary); block_end[i] = number of iters in blocks 0..i.
 *   axe_layout_tile          Alg. 2: T = A (x) B, f_T(x || y) = f_A(x) * span(B) + f_B(y); A and B
 *                            grouped by SA and SB (same rank); shape_out = (SA[0], SB[0], SA[1], ...),
 *                            2 * rank entries.  B may carry a swizzle stage if everything A adds on the
 *                            swizzled axis is a multiple of 2^(shift + bits) (else AXE_EUNSUPPORTED).
 *   axe_layout_direct_sum    App. F: as tile, without the span scaling: f(x || y) = f_A(x) + f_B(y).
 *   axe_layout_flatten       the layout on the single axis `to_axis` that L becomes when a coordinate c on axis a is
 *                            stored at sum_a c[a] * pitch[a] (pitch: n_axes entries): every iter (e, s @ a) of D and R
 *                            becomes (e, s * pitch[a] @ to_axis) (Def. 2.1), the offsets add up.  It turns a
 *                            thread-distributed layout (axes wave, lane, reg; Sec. 2.2) into the memory image
 *                            [wave][lane][reg] that axe_relayout can write: a register layout as relayout target.
 *                            Pitch 0 is allowed for axes that carry no iter of extent > 1; a swizzled L is
 *                            AXE_EUNSUPPORTED.
 *   axe_layout_tile_of       Alg. 3: decides A = C (x) B and recovers C; shape_out = SA / SB (rank entries).
 *   axe_layout_slice         Alg. 4: a layout admitting `size` with f(u) = f_{L<shape>}(begin + u); per
 *                            block the greedy peel, then the no-wrap or the symmetric one-wrap form.
 *                            A swizzle stage is kept (it acts on the sum D + R + O).
 */
int axe_layout_span(const axe_layout_t* L, int64_t* span);
int axe_layout_canonicalize(const axe_layout_t* L, axe_layout_t* out, void* arena, size_t arena_bytes);
int axe_layout_gap_condition(const axe_layout_t* L);
int axe_layout_equal(const axe_layout_t* A, const axe_layout_t* B);
int axe_layout_group(const axe_layout_t* L, int32_t rank, const int64_t* shape, axe_layout_t* out,
                     int32_t* block_end, void* arena, size_t arena_bytes);
int axe_layout_tile(const axe_layout_t* A, int32_t rank, const int64_t* SA, const axe_layout_t* B, const int64_t* SB,
                    axe_layout_t* out, int64_t* shape_out, void* arena, size_t arena_bytes);
int axe_layout_direct_sum(const axe_layout_t* A, int32_t rank, const int64_t* SA, const axe_layout_t* B,
                          const int64_t* SB, axe_layout_t* out, int64_t* shape_out, void* arena, size_t arena_bytes);
int axe_layout_flatten(const axe_layout_t* L, const int64_t* pitch, int32_t to_axis, axe_layout_t* out, void* arena,
                       size_t arena_bytes);
int axe_layout_tile_of(const axe_layout_t* A, int32_t rank, const int64_t* SA, const axe_layout_t* B, const int64_t* SB,
                       axe_layout_t* out, int64_t* shape_out, void* arena, size_t arena_bytes);
int axe_layout_slice(const axe_layout_t* L, int32_t rank, const int64_t* shape, const int64_t* begin,
                     const int64_t* size, axe_layout_t* out, void* arena, size_t arena_bytes);

const char* axe_strerror(int code);
const char* axe_last_error(void);
/* Library version: major * 10000 + minor * 100 + patch. */
int32_t axe_version(void);

#ifdef __cplusplus
}
#endif
#endif /* AXE_H */
