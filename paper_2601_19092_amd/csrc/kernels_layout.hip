// Integer kernels: layout evaluation (Def. 2.3) and relayout copies (`copy` operator, Sec. 3.2).
// gfx950 only.  Bandwidth-bound: no LDS, 128-bit global accesses wherever the layouts allow.
#include <hip/hip_runtime.h>

#include "device_types.h"
#include "kernels.h"

namespace axe {

__device__ __forceinline__ int64_t swz_apply(int64_t x, Swz z) {
  return x ^ (((x >> z.shift) & (int64_t)z.mask) << z.base);
}

// ------------------------------------------------------------------------------------------
// Layout evaluation: one thread per logical index.  Digits are peeled from the fastest iter
// (d_i = floor(x / p_i) mod e_i, App. A), each contributes digit * stride to its axis.
// ------------------------------------------------------------------------------------------
template <typename IdxT>
__global__ __launch_bounds__(256) void layout_eval_kernel(EvalDesc d, int64_t n, const int64_t* __restrict__ idx,
                                                          int64_t* __restrict__ out) {
  const int64_t per = d.E_R * d.n_axes;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    int64_t x = idx ? idx[i] : i;
    int64_t* o = out + i * per;
    if (x < 0 || x >= d.E_D) {
      for (int64_t t = 0; t < per; ++t) o[t] = INT64_MIN;
      continue;
    }
    int64_t c[kMaxAxes];
#pragma unroll
    for (int a = 0; a < kMaxAxes; ++a) c[a] = d.off[a];
    IdxT rem = (IdxT)x;
    for (int k = d.n_d - 1; k >= 0; --k) {
      IdxT e = (IdxT)d.ext[k];
      IdxT q = rem / e;
      int64_t v = (int64_t)(rem - q * e) * d.str[k];
      rem = q;
      int ax = d.axis[k];
#pragma unroll
      for (int a = 0; a < kMaxAxes; ++a) c[a] += (a == ax) ? v : 0;
    }
    for (int64_t t = 0; t < d.E_R; ++t) {
      int64_t r[kMaxAxes];
#pragma unroll
      for (int a = 0; a < kMaxAxes; ++a) r[a] = c[a];
      int64_t tr = t;
      for (int k = d.n_r - 1; k >= 0; --k) {
        int64_t q = tr / d.rext[k];
        int64_t v = (tr - q * d.rext[k]) * d.rstr[k];
        tr = q;
        int ax = d.raxis[k];
#pragma unroll
        for (int a = 0; a < kMaxAxes; ++a) r[a] += (a == ax) ? v : 0;
      }
#pragma unroll
      for (int a = 0; a < kMaxAxes; ++a) {
        if (a < d.n_axes) {
          int64_t v = r[a];
          if (a == d.swz_axis) v = swz_apply(v, d.swz);
          o[t * d.n_axes + a] = v;
        }
      }
    }
  }
}

// The common case -- no replicas, fewer than 2^31 points, at most 4 axes -- without the generic loop's
// 64-bit divisions and 8-way axis selects: digits in 32 bits (a shift and a mask where the extent is a
// power of two), one 64-bit multiply-add per digit, the axis loop unrolled to NAX.  A thread evaluates
// PTS consecutive indices (4 when there is a single axis: two 16-byte stores), so that an iter's
// parameters are fetched once for all of them.  Bound: the 8 NAX bytes written per index.
template <int NAX, int PTS>
__global__ __launch_bounds__(256) void layout_eval_fast_kernel(EvalDesc d, int64_t n, const int64_t* __restrict__ idx,
                                                               int64_t* __restrict__ out) {
  // index of the thread's p-th point: a wave owns 64 PTS consecutive indices; with one axis a lane takes pairs
  // (2 lane, 2 lane + 1) 128 apart, so that every store instruction of the wave writes 1 contiguous KiB;
  // otherwise lane-interleaved single indices (each store instruction 64 NAX x 8 contiguous bytes).
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int lane = (int)(t & 63);
  const int64_t wbase = (t >> 6) * (64 * PTS);
  auto index_of = [&](int p) -> int64_t {
    return (NAX == 1 && PTS % 2 == 0) ? wbase + (p >> 1) * 128 + lane * 2 + (p & 1) : wbase + p * 64 + lane;
  };
  if (wbase >= n) return;
  int64_t x[PTS], c[PTS][NAX];
  uint32_t rem[PTS];
#pragma unroll
  for (int p = 0; p < PTS; ++p) {
    const int64_t ip = index_of(p);
    const int64_t i = ip < n ? ip : n - 1;                         // (a ragged tail repeats the last index; not stored)
    x[p] = idx ? idx[i] : i;
    rem[p] = (uint32_t)x[p];
#pragma unroll
    for (int a = 0; a < NAX; ++a) c[p][a] = d.off[a];
  }
  // digits outermost: an iter's parameters are fetched once for the thread's PTS indices
  for (int k = d.n_d - 1; k >= 0; --k) {
    const int sh = d.shift[k];
    const uint32_t e = (uint32_t)d.ext[k];
    const int64_t st = d.str[k];
    const int ax = d.axis[k];
#pragma unroll
    for (int p = 0; p < PTS; ++p) {
      uint32_t dig;
      if (sh >= 0) {
        dig = rem[p] & (e - 1u);
        rem[p] >>= sh;
      } else {
        const uint32_t q = rem[p] / e;
        dig = rem[p] - q * e;
        rem[p] = q;
      }
      const int64_t v = (int64_t)dig * st;
      if (NAX == 1) {
        c[p][0] += v;
      } else {
#pragma unroll
        for (int a = 0; a < NAX; ++a) c[p][a] += (a == ax) ? v : 0;
      }
    }
  }
#pragma unroll
  for (int p = 0; p < PTS; ++p) {
    const bool bad = x[p] < 0 || x[p] >= d.E_D;
#pragma unroll
    for (int a = 0; a < NAX; ++a) {
      int64_t v = c[p][a];
      if (a == d.swz_axis) v = swz_apply(v, d.swz);
      c[p][a] = bad ? INT64_MIN : v;
    }
  }
  typedef __attribute__((ext_vector_type(2))) int64_t i64x2;
  if (NAX == 1 && PTS % 2 == 0) {                                  // out is 16-byte aligned (the host checks), the pair's first index is even
#pragma unroll
    for (int p = 0; p < PTS; p += 2) {
      const int64_t ip = index_of(p);
      if (ip + 1 < n) __builtin_nontemporal_store(i64x2{c[p][0], c[p + 1][0]}, (i64x2*)(out + ip));
      else if (ip < n) out[ip] = c[p][0];
    }
  } else {
#pragma unroll
    for (int p = 0; p < PTS; ++p) {
      const int64_t ip = index_of(p);
      if (ip < n) {
#pragma unroll
        for (int a = 0; a < NAX; ++a) __builtin_nontemporal_store(c[p][a], &out[ip * NAX + a]);
      }
    }
  }
}

hipError_t launch_layout_eval(const EvalDesc& d, int64_t n, const int64_t* idx, int64_t* out, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  if (d.use32 && d.E_R == 1 && d.n_r == 0 && d.n_axes <= 4 && n < (int64_t(1) << 40)) {
    const bool vec = d.n_axes == 1 && ((uintptr_t)out & 15) == 0;  // 4 indices per thread, two 16-byte stores
    const int pts = d.n_axes == 1 ? (vec ? 4 : 1) : 2;
    const int64_t threads = (n + pts - 1) / pts;
    const dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    switch (d.n_axes * 2 + (vec ? 1 : 0)) {
      case 3: hipLaunchKernelGGL((layout_eval_fast_kernel<1, 4>), grid, block, 0, s, d, n, idx, out); break;
      case 2: hipLaunchKernelGGL((layout_eval_fast_kernel<1, 1>), grid, block, 0, s, d, n, idx, out); break;
      case 4: hipLaunchKernelGGL((layout_eval_fast_kernel<2, 2>), grid, block, 0, s, d, n, idx, out); break;
      case 6: hipLaunchKernelGGL((layout_eval_fast_kernel<3, 2>), grid, block, 0, s, d, n, idx, out); break;
      default: hipLaunchKernelGGL((layout_eval_fast_kernel<4, 2>), grid, block, 0, s, d, n, idx, out); break;
    }
    return hipGetLastError();
  }
  int64_t blocks = (n + 255) / 256;
  if (blocks > 65536 * 4) blocks = 65536 * 4;
  if (d.use32)
    hipLaunchKernelGGL(layout_eval_kernel<uint32_t>, dim3((unsigned)blocks), dim3(256), 0, s, d, n, idx, out);
  else
    hipLaunchKernelGGL(layout_eval_kernel<uint64_t>, dim3((unsigned)blocks), dim3(256), 0, s, d, n, idx, out);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Relayout, joint loop nest.  Thread w decodes its digits (fastest first); its U unrolled
// elements step along one more digit.  All loads are issued before the first store.
// ------------------------------------------------------------------------------------------
template <int BYTES> struct Word;
template <> struct Word<1> { using T = uint8_t; };
template <> struct Word<2> { using T = uint16_t; };
template <> struct Word<4> { using T = uint32_t; };
template <> struct Word<8> { using T = __attribute__((ext_vector_type(2))) uint32_t; };
template <> struct Word<16> { using T = __attribute__((ext_vector_type(4))) uint32_t; };

template <int BYTES, int U, bool REPL, bool NT>
__global__ __launch_bounds__(256) void relayout_joint_kernel(RelayoutPlan p, const void* __restrict__ src_,
                                                             void* __restrict__ dst_) {
  using T = typename Word<BYTES>::T;
  const T* __restrict__ src = (const T*)src_;
  T* __restrict__ dst = (T*)dst_;
  uint64_t w64 = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (w64 >= p.threads) return;
  uint32_t w = (uint32_t)w64;            // host guarantees threads < 2^32
  int64_t s = p.s_off, d = p.d_off;
  for (int k = 0; k < p.n; ++k) {
    uint32_t dig;
    if (p.shift[k] >= 0) {
      dig = w & (p.ext[k] - 1);
      w >>= p.shift[k];
    } else {
      uint32_t q = w / p.ext[k];
      dig = w - q * p.ext[k];
      w = q;
    }
    s += (int64_t)dig * p.ss[k];
    d += (int64_t)dig * p.ds[k];
  }
  T v[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const T* a = &src[swz_apply(s + u * p.us, p.s_swz)];
    v[u] = NT ? __builtin_nontemporal_load(a) : *a;
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    int64_t da = d + u * p.ud;
    if (!REPL) {
      T* a = &dst[swz_apply(da, p.d_swz)];
      if (NT) __builtin_nontemporal_store(v[u], a);
      else *a = v[u];
    } else {
      for (int64_t t = 0; t < p.E_R; ++t) {
        int64_t tr = t, ra = da;
        for (int k = p.n_r - 1; k >= 0; --k) {
          int64_t q = tr / p.rext[k];
          ra += (tr - q * p.rext[k]) * p.rstr[k];
          tr = q;
        }
        dst[swz_apply(ra, p.d_swz)] = v[u];
      }
    }
  }
}

template <int BYTES, int U>
static hipError_t launch_joint_u(const RelayoutPlan& p, const void* src, void* dst, hipStream_t s) {
  unsigned blocks = (unsigned)((p.threads + 255) / 256);
  if (p.n_r > 0)
    hipLaunchKernelGGL((relayout_joint_kernel<BYTES, U, true, false>), dim3(blocks), dim3(256), 0, s, p, src, dst);
  else if (p.streaming)
    hipLaunchKernelGGL((relayout_joint_kernel<BYTES, U, false, true>), dim3(blocks), dim3(256), 0, s, p, src, dst);
  else
    hipLaunchKernelGGL((relayout_joint_kernel<BYTES, U, false, false>), dim3(blocks), dim3(256), 0, s, p, src, dst);
  return hipGetLastError();
}

template <int BYTES>
static hipError_t launch_joint_b(const RelayoutPlan& p, const void* src, void* dst, hipStream_t s) {
  switch (p.U) {
    case 1: return launch_joint_u<BYTES, 1>(p, src, dst, s);
    case 2: return launch_joint_u<BYTES, 2>(p, src, dst, s);
    case 4: return launch_joint_u<BYTES, 4>(p, src, dst, s);
    case 8: return launch_joint_u<BYTES, 8>(p, src, dst, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_relayout_joint(const RelayoutPlan& p, int unit_bytes, const void* src, void* dst, hipStream_t s) {
  if (p.threads == 0) return hipSuccess;
  switch (unit_bytes) {
    case 1: return launch_joint_b<1>(p, src, dst, s);
    case 2: return launch_joint_b<2>(p, src, dst, s);
    case 4: return launch_joint_b<4>(p, src, dst, s);
    case 8: return launch_joint_b<8>(p, src, dst, s);
    case 16: return launch_joint_b<16>(p, src, dst, s);
    default: return hipErrorInvalidValue;
  }
}

// ------------------------------------------------------------------------------------------
// Relayout, transposing: source and destination are contiguous along different digits of the joint
// loop nest (row-major <-> column-major and their batched, strided relatives).  Moving single
// elements would leave one side with 2-byte accesses scattered over rows; instead a workgroup
// takes a T x T tile of the two digits, reads it with 16-byte loads along the source-fast digit
// (T * EB = 128 to 512 contiguous bytes per tile row), parks it in LDS, and writes it with 16-byte
// stores along the destination-fast digit, each store gathering its 16 / EB elements from as many
// LDS rows.  The LDS image is XOR-swizzled, not padded: 16-byte chunk c of row r sits at chunk position
// c ^ (r / elements per chunk), which keeps the gather on distinct banks for every element size.
// ------------------------------------------------------------------------------------------
template <int EB, bool NT>
__global__ __launch_bounds__(256) void relayout_transpose_kernel(TransposePlan p, const uint8_t* __restrict__ src,
                                                                 uint8_t* __restrict__ dst) {
  constexpr int T = EB == 8 ? 64 : 128;                           // tile edge, elements (transpose_tile_edge)
  constexpr int CE = 16 / EB;                                    // elements per 16-byte chunk
  constexpr int CPR = T / CE;                                    // chunks per tile row
  constexpr int ROWB = T * EB;                                   // bytes of a tile row in LDS
  typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
  // LDS image of the tile: rows of ROWB bytes, the 16-byte chunk c of row r at chunk position c ^ (r / CE) -- the
  // same kind of XOR stage as the swizzled layouts of the GEMM tiles.  Rows come in whole chunks (one 16-byte
  // write each); on the way out a lane gathers the CE elements of its chunk from CE consecutive rows at one
  // column, and the 16 (or more) lanes that do so for neighbouring chunks sit CE rows apart: their keys differ,
  // so they read different banks (a padded pitch cannot do that for 1- and 2-byte elements: CE x pitch is a
  // multiple of 8 words, and two of every 16 lanes met in a bank).  Measured: the conflict counter drops to
  // zero.
  __shared__ __attribute__((aligned(16))) uint8_t tile[T * ROWB];
  auto lds_at = [&](int row, int byte_col, int key) -> uint8_t* {
    return tile + row * ROWB + ((((byte_col >> 4) ^ key) & (CPR - 1)) << 4) + (byte_col & 15);
  };

  // workgroup -> (tile along S, tile along D, outer digits)
  uint64_t b = blockIdx.x;
  const uint32_t ts = (uint32_t)(b % p.tiles_s);
  b /= p.tiles_s;
  uint32_t td = (uint32_t)(b % p.tiles_d);
  b /= p.tiles_d;
  // Row by row (ts fastest, td fixed for tiles_s workgroups in a row) the workgroups running at one time read
  // whole rows of the source between them, but write one narrow column of the destination: short segments a row
  // pitch apart, which with power-of-two pitches fall on a fraction of the memory channels.  Walking the tiles
  // diagonally gives every window of workgroups many different td as well as many different ts.
  if (p.diag > 0) td = (td + ts / (uint32_t)p.diag) % p.tiles_d;
  int64_t sb = p.s_off, db = p.d_off;
  for (int k = 0; k < p.n; ++k) {
    const uint64_t q = b / p.ext[k];
    const int64_t dig = (int64_t)(b - q * p.ext[k]);
    sb += dig * p.ss[k];
    db += dig * p.ds[k];
    b = q;
  }
  const int64_t s0 = (int64_t)ts * T, d0 = (int64_t)td * T;      // tile origin in the two digits

  // HBM -> LDS: row r of the tile is destination-fast index d0 + r, its chunks run along the source.  All loads
  // of a thread are issued before the first of them is waited for: with one load at a time in flight per thread
  // the kernel was bound by the latency of HBM (4.1 - 4.2 TB/s on 8192 x 8192 bf16, whatever the LDS layout or the
  // order of the tiles), not by its bandwidth.
  constexpr int NL = T * CPR / 256;                              // chunks per thread
  u32x4 held[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int c = (int)threadIdx.x + 256 * i;
    const int r = c / CPR, cc = c % CPR;
    const int64_t iD = d0 + r, iS = s0 + (int64_t)cc * CE;
    // extents are multiples of CE: a chunk is in or out as a whole.  A chunk outside the tensor is replaced by the
    // tile's first one (always inside) instead of being skipped: a load under a branch would be waited for at
    // the end of that branch, one by one.
    const bool in = iD < p.eD && iS < p.eS;
    // (a swizzle stage moves whole chunks: the host admits it here only when it leaves the bits inside a chunk alone)
    const u32x4* a = (const u32x4*)(src + swz_apply(sb + (in ? iD * p.sD + iS : d0 * p.sD + s0), p.s_swz) * EB);
    held[i] = NT ? __builtin_nontemporal_load(a) : *a;
  }
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int c = (int)threadIdx.x + 256 * i;
    const int r = c / CPR, cc = c % CPR;
    *(u32x4*)lds_at(r, cc * 16, r / CE) = held[i];               // (chunks outside the tensor: values nobody reads)
  }
  __syncthreads();
  // LDS -> HBM: output row r is source-fast index s0 + r, its chunks run along the destination
  for (int c = threadIdx.x; c < T * CPR; c += 256) {
    const int r = c / CPR, cc = c % CPR;
    const int64_t iS = s0 + r, iD = d0 + (int64_t)cc * CE;
    if (iS < p.eS && iD < p.eD) {
      // element k of the chunk: LDS row cc * CE + k (key cc), column r
      u32x4 v;
      if (EB == 1) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          uint32_t w = 0;
#pragma unroll
          for (int k = 0; k < 4; ++k) w |= (uint32_t)*lds_at(cc * CE + 4 * j + k, r, cc) << (8 * k);
          v[j] = w;
        }
      } else if (EB == 2) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t lo = *(const uint16_t*)lds_at(cc * CE + 2 * j, r * 2, cc);
          const uint32_t hi = *(const uint16_t*)lds_at(cc * CE + 2 * j + 1, r * 2, cc);
          v[j] = lo | (hi << 16);
        }
      } else if (EB == 4) {
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = *(const uint32_t*)lds_at(cc * CE + j, r * 4, cc);
      } else {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          const uint32_t* q = (const uint32_t*)lds_at(cc * CE + j, r * 8, cc);
          v[2 * j] = q[0];
          v[2 * j + 1] = q[1];
        }
      }
      for (int64_t t = 0; t < p.E_R; ++t) {                        // every replica of the destination (usually one)
        int64_t tr = t, ra = db + iS * p.dS + iD;
        for (int k = p.n_r - 1; k >= 0; --k) {
          ra += (tr % p.rext[k]) * p.rstr[k];
          tr /= p.rext[k];
        }
        u32x4* a = (u32x4*)(dst + swz_apply(ra, p.d_swz) * EB);
        if (NT) __builtin_nontemporal_store(v, a);
        else *a = v;
      }
    }
  }
}

// The same transposition element by element, for pairs of layouts the 16-byte variant cannot take: extents, strides
// or offsets that are no multiples of a chunk, buffers that are not 16-byte aligned, a swizzle that reaches into a
// chunk.  A workgroup moves a 64 x 64 tile: each wave instruction reads 64 consecutive elements along the
// source-fast digit and writes 64 consecutive elements along the destination-fast digit (the per-element kernel
// leaves one side with single elements scattered over rows); the tile is parked in LDS with a pitch of 65 words.
template <int EB>
__global__ __launch_bounds__(256) void relayout_transpose_elem_kernel(TransposePlan p, const void* __restrict__ src_,
                                                                      void* __restrict__ dst_) {
  constexpr int T = 64;
  using W = typename Word<EB>::T;
  const W* __restrict__ src = (const W*)src_;
  W* __restrict__ dst = (W*)dst_;
  __shared__ W tile[T][T + 1];
  uint64_t b = blockIdx.x;
  const uint32_t ts = (uint32_t)(b % p.tiles_s);
  b /= p.tiles_s;
  uint32_t td = (uint32_t)(b % p.tiles_d);
  b /= p.tiles_d;
  if (p.diag > 0) td = (td + ts / (uint32_t)p.diag) % p.tiles_d;
  int64_t sb = p.s_off, db = p.d_off;
  for (int k = 0; k < p.n; ++k) {
    const uint64_t q = b / p.ext[k];
    const int64_t dig = (int64_t)(b - q * p.ext[k]);
    sb += dig * p.ss[k];
    db += dig * p.ds[k];
    b = q;
  }
  const int64_t s0 = (int64_t)ts * T, d0 = (int64_t)td * T;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  // tile row r: destination-fast index d0 + r, lanes along the source.  All 16 loads of a thread are issued before
  // the first is used (an element outside the tensor is replaced by the tile's first one, always inside: a load
  // under a branch would be waited for at the end of that branch, one by one)
  W held[T / 4];
#pragma unroll
  for (int k = 0; k < T / 4; ++k) {
    const int64_t iD = d0 + ty + 4 * k, iS = s0 + tx;
    const bool in = iD < p.eD && iS < p.eS;
    held[k] = src[swz_apply(sb + (in ? iD * p.sD + iS : d0 * p.sD + s0), p.s_swz)];
  }
#pragma unroll
  for (int k = 0; k < T / 4; ++k) tile[ty + 4 * k][tx] = held[k];
  __syncthreads();
  for (int r = ty; r < T; r += 4) {                              // output row r: source-fast index s0 + r, lanes along the destination
    const int64_t iS = s0 + r, iD = d0 + tx;
    if (iS < p.eS && iD < p.eD) {
      const W v = tile[tx][r];
      for (int64_t t = 0; t < p.E_R; ++t) {
        int64_t tr = t, ra = db + iS * p.dS + iD;
        for (int k = p.n_r - 1; k >= 0; --k) {
          ra += (tr % p.rext[k]) * p.rstr[k];
          tr /= p.rext[k];
        }
        dst[swz_apply(ra, p.d_swz)] = v;               // (ordinary stores: single elements written non-temporally do not combine -- 3.8 -> 1.7 TB/s on bf16)
      }
    }
  }
}

template <int EB>
static hipError_t launch_transpose_e(const TransposePlan& p, const void* src, void* dst, hipStream_t s) {
  if (p.streaming)
    hipLaunchKernelGGL((relayout_transpose_kernel<EB, true>), dim3((unsigned)p.blocks), dim3(256), 0, s, p, (const uint8_t*)src,
                       (uint8_t*)dst);
  else
    hipLaunchKernelGGL((relayout_transpose_kernel<EB, false>), dim3((unsigned)p.blocks), dim3(256), 0, s, p, (const uint8_t*)src,
                       (uint8_t*)dst);
  return hipGetLastError();
}

hipError_t launch_relayout_transpose(const TransposePlan& p, int elem_bytes, const void* src, void* dst, hipStream_t s) {
  if (p.blocks == 0) return hipSuccess;
  if (p.blocks > 0x7fffffffull) return hipErrorInvalidValue;
  if (p.elementwise) {
    const dim3 grid((unsigned)p.blocks), block(256);
    switch (elem_bytes) {
      case 1: hipLaunchKernelGGL(relayout_transpose_elem_kernel<1>, grid, block, 0, s, p, src, dst); break;
      case 2: hipLaunchKernelGGL(relayout_transpose_elem_kernel<2>, grid, block, 0, s, p, src, dst); break;
      case 4: hipLaunchKernelGGL(relayout_transpose_elem_kernel<4>, grid, block, 0, s, p, src, dst); break;
      case 8: hipLaunchKernelGGL(relayout_transpose_elem_kernel<8>, grid, block, 0, s, p, src, dst); break;
      default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
  }
  switch (elem_bytes) {
    case 1: return launch_transpose_e<1>(p, src, dst, s);
    case 2: return launch_transpose_e<2>(p, src, dst, s);
    case 4: return launch_transpose_e<4>(p, src, dst, s);
    case 8: return launch_transpose_e<8>(p, src, dst, s);
    default: return hipErrorInvalidValue;
  }
}

// ------------------------------------------------------------------------------------------
// Relayout, generic: one element per thread, source and destination decoded separately from
// the logical index.  Correct for any pair of layouts; used when no joint loop nest exists.
// ------------------------------------------------------------------------------------------
template <int BYTES>
__global__ __launch_bounds__(256) void relayout_generic_kernel(GenericRelayoutPlan p, const void* __restrict__ src_,
                                                               void* __restrict__ dst_) {
  using T = typename Word<BYTES>::T;
  const T* __restrict__ src = (const T*)src_;
  T* __restrict__ dst = (T*)dst_;
  for (int64_t x = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; x < p.total; x += (int64_t)gridDim.x * blockDim.x) {
    int64_t s = p.s_off, d = p.d_off;
    uint64_t rem = (uint64_t)x;
    for (int k = p.ns - 1; k >= 0; --k) {
      uint64_t q = rem / (uint64_t)p.sext[k];
      s += (int64_t)(rem - q * (uint64_t)p.sext[k]) * p.sstr[k];
      rem = q;
    }
    rem = (uint64_t)x;
    for (int k = p.nd - 1; k >= 0; --k) {
      uint64_t q = rem / (uint64_t)p.dext[k];
      d += (int64_t)(rem - q * (uint64_t)p.dext[k]) * p.dstr[k];
      rem = q;
    }
    T v = src[swz_apply(s, p.s_swz)];
    for (int64_t t = 0; t < p.E_R; ++t) {
      int64_t tr = t, ra = d;
      for (int k = p.n_r - 1; k >= 0; --k) {
        int64_t q = tr / p.rext[k];
        ra += (tr - q * p.rext[k]) * p.rstr[k];
        tr = q;
      }
      dst[swz_apply(ra, p.d_swz)] = v;
    }
  }
}

hipError_t launch_relayout_generic(const GenericRelayoutPlan& p, int unit_bytes, const void* src, void* dst,
                                   hipStream_t s) {
  if (p.total <= 0) return hipSuccess;
  int64_t blocks = (p.total + 255) / 256;
  if (blocks > 65536 * 4) blocks = 65536 * 4;
  dim3 g((unsigned)blocks), b(256);
  switch (unit_bytes) {
    case 1: hipLaunchKernelGGL(relayout_generic_kernel<1>, g, b, 0, s, p, src, dst); break;
    case 2: hipLaunchKernelGGL(relayout_generic_kernel<2>, g, b, 0, s, p, src, dst); break;
    case 4: hipLaunchKernelGGL(relayout_generic_kernel<4>, g, b, 0, s, p, src, dst); break;
    case 8: hipLaunchKernelGGL(relayout_generic_kernel<8>, g, b, 0, s, p, src, dst); break;
    case 16: hipLaunchKernelGGL(relayout_generic_kernel<16>, g, b, 0, s, p, src, dst); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace axe
