// WtdAttn (Alg. 3) and the query radius R_Q of Alg. 4 for gfx950.
//
// WtdAttn is flash-attention shaped with a key length of only r: per query tile the coreset is streamed
// through LDS once, scores and the value product run on MFMA with fp32 accumulation, and a running
// maximum keeps exp() in range.  Any positive per-row factor cancels in Alg. 3's ratio and leaves the
// sign of the normaliser (A w) unchanged, so the max shift does not alter the "> 0" guard.
//
// Kernels:
//   k_wtd_attn_mfma2    bf16 storage with packed values (coreset fields v_t, v_scale), d and dv of 64 or 128 (and
//                       64 / 256): transposed tiles on v_mfma_f32_32x32x16, pipelined through LDS.
//   k_wtd_attn_decode   the same arithmetic at decode shape (few queries per head): the key tiles are dealt out to
//                       the waves of a workgroup, operands straight from memory.
//   k_wtd_attn_mfma_f32 fp32 storage (d / dv of 64 / 64, 64 / 256, 128 / 128) on v_mfma_f32_32x32x2_f32.
//   k_wtd_attn_f32_split  the same at few queries in all (dv <= 128): the waves of a workgroup share one block of 32
//                       queries and split its key tiles, operands straight from memory.
//   k_wtd_attn_simple   any storage type / width, fp32 arithmetic on the vector ALU (what the MFMA kernels do
//                       not cover).
//   k_qnorm_max(_vec), k_radius_final   the query radius R_Q;   k_value_scale, k_pack_values   the packed values.
#include <atomic>
#include <climits>
#include <cmath>

#include "common.h"

namespace wildcat {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr float kLog2e = 1.4426950408889634f;

// --------------------------------------------------------------------------------------------
// R_Q = max over the rows of all query heads sharing a kv head of ||q||_2 (Alg. 4, second line).
// Squared norms in fp64; the maximum of non-negative doubles is taken on their bit patterns with an
// integer atomic (exact, order-independent).  grid (ceil(m/256), batch*q_heads).
// --------------------------------------------------------------------------------------------
__global__ void k_zero_u64(unsigned long long *x, int count) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) x[i] = 0ull;
}

// The accumulator holds the bit pattern of the largest norm so far (sqrt is monotone and correctly rounded, so the
// largest norm is the root of the largest squared norm).  It only grows: a workgroup whose maximum is not above
// what is already there skips the contended atomic (a stale read merely costs an atomic that changes nothing).
__device__ __forceinline__ void publish_radius(unsigned long long *acc, double max_sq) {
  const unsigned long long bits = (unsigned long long)__double_as_longlong(sqrt(max_sq));
  if (bits > __hip_atomic_load(acc, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) atomicMax(acc, bits);
}

// Generic version: one thread per query row.
template <typename T>
__global__ __launch_bounds__(kThreads) void k_qnorm_max(const T *__restrict__ Q, int64_t m, int d, int q_heads,
                                                        int group, unsigned long long *__restrict__ acc) {
  __shared__ double sm[kThreads / kWave];
  const int bh = blockIdx.y;
  const int b = bh / q_heads, hq = bh % q_heads;
  const int pr = b * (q_heads / group) + hq / group;
  const int64_t row = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  double s = 0.0;
  if (row < m) {
    const T *q = Q + ((size_t)bh * m + row) * d;
    for (int j = 0; j < d; ++j) {
      const double v = (double)to_float(q[j]);
      s = fma(v, v, s);
    }
  }
  s = block_reduce<double>(s, sm, MaxOp());
  if (threadIdx.x == 0) publish_radius(&acc[pr], s);
}

// Coalesced version for rows that are a power-of-two number (<= 64) of 16-byte pieces: LPR lanes share a
// row, each loads one 16-byte piece, squares are summed in fp64 and combined with a butterfly over the
// LPR lanes.  grid (blocks, batch*q_heads); each workgroup walks rows blockIdx.x*rpb .. with stride.
__device__ __forceinline__ double sumsq16(const uint4 v, float) {
  const float x[4] = {__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w)};
  double s = 0.0;
#pragma unroll
  for (int e = 0; e < 4; ++e) s = fma((double)x[e], (double)x[e], s);
  return s;
}
__device__ __forceinline__ double sumsq16(const uint4 v, bf16_t) {
  const unsigned int wds[4] = {v.x, v.y, v.z, v.w};
  double s = 0.0;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const double lo = (double)__uint_as_float(wds[e] << 16), hi = (double)__uint_as_float(wds[e] & 0xffff0000u);
    s = fma(lo, lo, s);
    s = fma(hi, hi, s);
  }
  return s;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void k_qnorm_max_vec(const T *__restrict__ Q, int64_t m, int d, int lpr,
                                                            int q_heads, int group,
                                                            unsigned long long *__restrict__ acc,
                                                            double *__restrict__ partial) {
  __shared__ double sm[kThreads / kWave];
  const int bh = blockIdx.y;
  const int b = bh / q_heads, hq = bh % q_heads;
  const int pr = b * (q_heads / group) + hq / group;
  const int rows_per_pass = kThreads / lpr;
  const int sub = threadIdx.x % lpr, rloc = threadIdx.x / lpr;
  const uint4 *base = reinterpret_cast<const uint4 *>(Q + (size_t)bh * m * d);
  double best = 0.0;
  const int64_t stride = (int64_t)gridDim.x * rows_per_pass;
  for (int64_t row0 = (int64_t)blockIdx.x * rows_per_pass + rloc; row0 < m; row0 += 4 * stride) {
    uint4 v[4];                                            // four rows in flight per thread
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t row = row0 + q * stride;
      v[q] = row < m ? base[row * lpr + sub] : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      double s = sumsq16(v[q], T());
      for (int off = lpr / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, kWave);
      best = fmax(best, s);
    }
  }
  best = block_reduce<double>(best, sm, MaxOp());
  if (threadIdx.x == 0) {
    if (partial) partial[(size_t)bh * gridDim.x + blockIdx.x] = best;     // combined by k_radius_final
    else publish_radius(&acc[pr], best);
  }
}

// Second stage when scratch memory is available: thousands of atomics on a handful of addresses serialise (they
// cost more than reading Q), plain per-workgroup results combined here do not.  grid P; `count` = group * blocks
// consecutive partial maxima of squared norms belong to one kv head.
__global__ __launch_bounds__(kThreads) void k_radius_final(const double *__restrict__ partial, int count,
                                                           double *__restrict__ r_q_out) {
  __shared__ double sm[kThreads / kWave];
  const int pr = blockIdx.x;
  double best = 0.0;
  for (int e = threadIdx.x; e < count; e += kThreads) best = fmax(best, partial[(size_t)pr * count + e]);
  best = block_reduce<double>(best, sm, MaxOp());
  if (threadIdx.x == 0) r_q_out[pr] = sqrt(best);
}

// --------------------------------------------------------------------------------------------
// Generic fp32 kernel.  Workgroup = 16 queries x 16 threads; key tiles of 16 through LDS.
// --------------------------------------------------------------------------------------------
constexpr int kSQ = 16, kSK = 16;

template <typename T>
__global__ __launch_bounds__(kThreads) void k_wtd_attn_simple(const T *__restrict__ Q, const T *__restrict__ Ks,
                                                              const float *__restrict__ Vs, const float *__restrict__ w,
                                                              const float *__restrict__ vmin,
                                                              const float *__restrict__ vmax,
                                                              const int32_t *__restrict__ r_eff, T *__restrict__ out,
                                                              int64_t m, int d, int dv, int r, int q_heads, int group,
                                                              float beta) {
  extern __shared__ float lds[];
  float *sq = lds;                       // [16][d+1]
  float *sk = sq + kSQ * (d + 1);        // [16][d+1]
  float *sv = sk + kSK * (d + 1);        // [16][dv]
  float *sw = sv + kSK * dv;             // [16]
  float *sp = sw + kSK;                  // [16][16]
  const int t = threadIdx.x, qi = t / 16, sub = t % 16;
  const int bh = blockIdx.y, b = bh / q_heads, hq = bh % q_heads;
  const int pr = b * (q_heads / group) + hq / group;
  const int64_t q0 = (int64_t)blockIdx.x * kSQ;
  const int re = r_eff ? min(r_eff[pr], r) : r;
  for (int e = t; e < kSQ * d; e += kThreads) {
    const int qq = e / d, j = e % d;
    const int64_t row = q0 + qq < m ? q0 + qq : m - 1;
    sq[qq * (d + 1) + j] = to_float(Q[((size_t)bh * m + row) * d + j]);
  }
  constexpr int kMaxCols = kMaxWidth / 16;
  float acc[kMaxCols];
#pragma unroll
  for (int c = 0; c < kMaxCols; ++c) acc[c] = 0.0f;
  float mrun = -INFINITY, den = 0.0f;
  for (int k0 = 0; k0 < re; k0 += kSK) {
    __syncthreads();
    for (int e = t; e < kSK * d; e += kThreads) {
      const int kk = e / d, j = e % d;
      sk[kk * (d + 1) + j] = k0 + kk < re ? to_float(Ks[((size_t)pr * r + k0 + kk) * d + j]) : 0.0f;
    }
    for (int e = t; e < kSK * dv; e += kThreads) {
      const int kk = e / dv;
      sv[e] = k0 + kk < re ? Vs[((size_t)pr * r + k0 + kk) * dv + (e % dv)] : 0.0f;
    }
    if (t < kSK) sw[t] = k0 + t < re ? w[(size_t)pr * r + k0 + t] : 0.0f;
    __syncthreads();
    float s0 = 0.0f;
    for (int j = 0; j < d; ++j) s0 = fmaf(sq[qi * (d + 1) + j], sk[sub * (d + 1) + j], s0);
    s0 = k0 + sub < re ? s0 * beta : -INFINITY;
    float mx = s0;
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 16));
    const float mnew = fmaxf(mrun, mx);
    const float alpha = expf(mrun - mnew);
    const float p0 = expf(s0 - mnew);
    sp[qi * kSK + sub] = p0;
    float dl = p0 * sw[sub];
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) dl += __shfl_xor(dl, off, 16);
    den = den * alpha + dl;
    mrun = mnew;
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kMaxCols; ++c) {
      const int col = sub + 16 * c;
      if (col < dv) {
        float a = acc[c] * alpha;
        for (int kk = 0; kk < kSK; ++kk) a = fmaf(sp[qi * kSK + kk], sv[kk * dv + col], a);
        acc[c] = a;
      }
    }
  }
  if (q0 + qi < m) {
    const float inv = den > 0.0f ? 1.0f / den : 0.0f;
#pragma unroll
    for (int c = 0; c < kMaxCols; ++c) {
      const int col = sub + 16 * c;
      if (col < dv) {
        float o = den > 0.0f ? acc[c] * inv : 0.0f;
        o = fminf(fmaxf(o, vmin[(size_t)pr * dv + col]), vmax[(size_t)pr * dv + col]);
        from_float(o, &out[((size_t)bh * m + q0 + qi) * dv + col]);
      }
    }
  }
}

// --------------------------------------------------------------------------------------------
// MFMA kernel for bf16 storage (needs the packed half-precision values v_t of the coreset).
//
// v_mfma_f32_32x32x16_{bf16,f16} operand layout (lane l, g = l / 32):
//   A (32 x 16): row l % 32, k = 8 g .. 8 g + 7        B (16 x 32): column l % 32, k = 8 g .. 8 g + 7
//   D (32 x 32): column l % 32, register v holds row 8 (v / 4) + 4 g + (v % 4)
// The kernel works on transposed tiles so that all softmax state of a query lives in one lane pair:
// S^T = K_S Q^T (bf16 operands) and O^T = V_S^T P^T.  In an S^T tile rows = keys and columns = queries, so lane l
// holds 16 key scores of query l % 32 and lane l ^ 32 the other 16.  Registers 8h .. 8h+7 of such a tile, converted
// to half precision, are used directly as the B operand of the value product.  They are rows
// {16h + 4g + 0..3, 16h + 8 + 4g + 0..3} of the tile; so that they are the eight CONSECUTIVE keys 16h + 8g + 0..7
// that lane group g must supply (and one 16-byte LDS read fetches the matching piece of V_S^T), the key tile is
// stored with its rows permuted: LDS row rho holds key pi(rho) = rho with bits 2 and 3 exchanged (softmax does
// not care in which order it sees the keys; only the loads, the weights and the ragged-tile mask follow pi).
//
// The value product runs on fp16 operands, not bf16.  Nystrom weights have both signs, so numerator and normaliser
// of Alg. 3 can be far smaller than the sum of the magnitudes of their terms (hundreds of times for some queries of
// the long-context workload); operand rounding is relative to the terms, and the 8-bit significand of bf16 then
// costs several per cent of the output range.  fp16 carries 11 bits at the same MFMA rate.  Its narrow exponent is
// handled by construction: P lies in (0, 2^8] with the row maximum >= 1 (see below), and v_t stores V_S^T divided
// by a per-problem power of two (coreset field v_scale) that is multiplied back in the epilogue.  The normaliser
// sum_s P_s w_s is accumulated in fp32 on the vector ALU from the unrounded P: with weights of both signs it can be
// hundreds of times smaller than its terms, and P rounded to half precision then costs a tenth of the output range
// on the long-context workload (measured, with the sum taken on the matrix unit from the rounded P and the weights
// in three half-precision parts).
//
// Workgroup = NW wavefronts (eight), each owning 32 queries; two
// waves per SIMD, so that one wave's exp/convert work overlaps another's MFMAs.  Key tiles of 64 are
// double-buffered in LDS.  While tile t is computed, the global loads of tile t+2 fly into a few staging
// registers (each wave fetches 1 KB pieces: lane i holds bytes 16 i .. 16 i + 15); at the start of tile t+1 they
// are stored into the buffer tile t was read from.  So a tile's loads have a whole tile time to arrive -- under
// load the trip to L2 and back takes about that long -- and the wait for them is an ordinary register dependence.
// (Direct global-to-LDS loads, which need no staging registers, were measured and dropped: while one is in flight
// the compiler turns every wait for an LDS operand into a wait for ALL outstanding LDS reads, which rules out
// requesting operands ahead of the MFMAs that use them.)  One barrier per tile.
//
// LDS rows are padded by one 16-byte piece (key rows 2 d + 16 bytes, value-column rows 144): sixteen consecutive
// rows then put the same piece into sixteen different 16-byte bank groups, and a lane's operand addresses are one
// base plus compile-time offsets.
//
// The running maximum is only a reference point for exp(): any reference within 2^8 of the true row maximum
// keeps every exponential in range, and a change of reference multiplies numerator and normaliser of a row
// alike.  So the accumulators are rescaled only when a row's maximum has grown by more than 8 (log2 units)
// since its reference was set -- rare after the first tile -- instead of on every tile.  The reference is always
// a maximum the row has already seen, so the largest P of a row is >= 1 and every P is <= 2^8.
// --------------------------------------------------------------------------------------------
constexpr int kKT = 64;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr float kRescaleSlack = 8.0f;
constexpr int kSchedMfma = 0x008, kSchedDsRead = 0x100;      // instruction classes of sched_group_barrier
// Maximum / sum of x over the lane pair {l, l ^ 32}.  The lane-half swap instruction applied to (x, x) returns
// (lower half of x in both halves, upper half of x in both halves): no trip through the LDS crossbar, which a
// shuffle would take.
__device__ __forceinline__ float pair_max(float x) {
  const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
}

// Wavefronts per workgroup: eight, two per SIMD (against four, a wave fetches half as many pieces per tile and each
// tile serves twice the queries).
template <int D, int DV>
constexpr int attn_waves() { return 8; }


// A 64-key tile of an item: item = (batch*head, query tile) pair, pr its coreset, re the number of filled slots,
// k0 the first key of the tile.  item >= total_items marks the end of the workgroup's list; pr, re and k0 then
// still name a valid tile (loads of it are harmless and never used).
struct TilePos {
  int item, pr, re, k0;
};

// Kernel arguments and per-wave state of the pipelined kernel, passed by reference to the per-tile function.
template <int D, int DV, int NW>
struct AttnCtx {
  const bf16_t *Q, *Ks;
  const uint16_t *Vt;         // fp16 bit patterns
  const float *w, *vmin, *vmax, *vscale;
  const int32_t *r_eff;
  bf16_t *out;
  int64_t m;
  int r, r64, q_heads, group, kv_heads, qtiles, total_items, stride;
  float scale_log2;
  int wv, l, g, c32;
  uint32_t kst, vst;          // byte offsets of this lane's first piece in the key / value tile of an LDS buffer
  uint32_t kop, vop;          // ... of its MFMA operands: row c32 of the key (value) tile, piece g
  // per-lane byte offsets of this wave's tile loads from the tile's first key row / first value column entry
  // (fixed for the whole kernel; the tile's own address is wave-uniform and stays in scalar registers)
  // this lane's piece 0: key row and byte in the row; byte offset in the value tile (piece e: KROWS_PER_LOAD rows,
  // VROWS_PER_LOAD value columns further on)
  uint32_t krow, kcol, voff;
  // This wave's small piece of a tile (all wave-uniform): CW floats at sm_base + pr * sm_stride + k0 * sm_tile,
  // stored at byte sm_dst of the buffer (the second 64, where CW = 128, at sm_dst2).  Wave 0 carries the tile's 64
  // weights, waves 1 .. CLOADS CW entries of v_min | v_max each (so every buffer holds the clip vectors of its
  // tile's problem); the other waves load the weights too and drop them into a spare corner, which keeps the tile
  // code free of branches.
  const float *sm_base;
  const float *sm_cap;        // entries of v_min are stored as min(v_min, v_max): sm_cap = the matching entries of v_max; else = sm_base
  int sm_stride, sm_tile, sm_dst, sm_dst2;
  // state: the tile being computed and the one after it, whose data is in the staging registers (or on its way)
  TilePos cur, nxt;
  u32x4 stage[(kKT * (D / 8) + DV * (kKT / 8)) / 64 / NW];   // this wave's 1 KB pieces of tile nxt
  float stage_small, stage_small2;   // wave 0: weight of key l of tile nxt; waves 1 .. CLOADS: entries of v_min | v_max
  bf16x8 qf[D / 16];          // Q fragments: B operand of S^T = K Q^T (query c32, features 16 kb + 8 g .. + 7)
  floatx16 acc[DV / 32];      // O^T accumulators
  float mref, den;            // reference exponent (log2 domain) and normaliser of query c32
  float vsc, nvsc;            // v_scale of this item's problem and of the next item's
};

template <int D, int DV, int NW>
struct AttnGeom {
  static constexpr int KPPR = D / 8;                     // 16-byte pieces per key row
  static constexpr int VPPR = kKT / 8;                   // 16-byte pieces per value-column row (= 8)
  static constexpr int KLOADS = kKT * KPPR / 64 / NW;    // wave-wide 1 KB loads of the key tile per wave
  static constexpr int VLOADS = DV * VPPR / 64 / NW;     // ... of the value tile
  static constexpr int CW = 2 * DV / 64 <= NW - 1 ? 64 : 128;   // clip entries a wave carries per tile
  static constexpr int CLOADS = 2 * DV / CW;             // waves that carry clip entries
  static_assert(KLOADS * NW * 64 == kKT * KPPR && VLOADS * NW * 64 == DV * VPPR, "tiles must split evenly");
  static_assert(DV % 32 == 0 && CLOADS <= NW - 1, "clip vectors are loaded by waves 1 .. CLOADS");
  // One LDS buffer (bytes): key tile | value tile | weights | clip vectors (v_min | v_max)
  static constexpr int KROWB = 2 * D + 16;               // bytes of a key row in LDS (padded by one piece)
  static constexpr int VROWB = 2 * kKT + 16;             // bytes of a value-column row in LDS (padded likewise)
  static constexpr int KROWS_PER_LOAD = NW * 64 / KPPR;  // key rows (value rows) that the workgroup's pieces e and e + 1 lie apart
  static constexpr int VROWS_PER_LOAD = NW * 64 / VPPR;
  static constexpr int OFF_K = 0;
  static constexpr int OFF_V = OFF_K + kKT * KROWB;
  static constexpr int OFF_W = OFF_V + DV * VROWB;
  static constexpr int OFF_C = OFF_W + kKT * 4;
  static constexpr int OFF_SPARE = OFF_C + 2 * DV * 4;     // where waves without a small piece of their own write
  static constexpr int BYTES = OFF_SPARE + 512;
  static constexpr int OROWB = 64 * 2 + 16;                // bytes of a row of the output staging area (padded)
  static constexpr int OBYTES = NW * 32 * OROWB;
  static constexpr int LPF = KLOADS + VLOADS;            // a wave's 1 KB pieces per tile
};

template <int D, int DV, int NW>
__device__ __forceinline__ int attn_item_pr(const AttnCtx<D, DV, NW> &c, int item) {
  const int bh = item / c.qtiles;
  return (bh / c.q_heads) * c.kv_heads + (bh % c.q_heads) / c.group;
}
template <int D, int DV, int NW>
__device__ __forceinline__ int attn_item_re(const AttnCtx<D, DV, NW> &c, int pr) {
  return c.r_eff ? max(min(c.r_eff[pr], c.r), 1) : c.r;      // never below 1: the tile loads clamp rows to re - 1
}
// The tile after p in this workgroup's list: the next tile of the item, else tile 0 of item + gridDim.x.
template <int D, int DV, int NW>
__device__ __forceinline__ TilePos attn_advance(const AttnCtx<D, DV, NW> &c, const TilePos p) {
  TilePos n = p;
  const bool within = p.k0 + kKT < p.re;
  n.k0 = within ? p.k0 + kKT : 0;
  if (!within && p.item < c.total_items) {                    // once per item
    n.item = p.item + c.stride;
    if (n.item < c.total_items) {
      n.pr = attn_item_pr(c, n.item);
      n.re = attn_item_re(c, n.pr);
    }
  }
  return n;
}

// Global loads of one tile into the staging registers.  A tile's address is wave-uniform (scalar registers); each
// lane adds an offset that was worked out once (AttnCtx::krow, kcol, voff).  In a ragged last tile (fewer than 64
// rows left in the coreset) the rows are clamped to the last one -- by a minimum that is a no-op in full tiles --
// and the clamped rows are masked after the score product.  v_t is zero padded to a multiple of 64 columns.  The
// first KLOADS pieces are 1 KB of keys each, the rest 1 KB of values; for the small piece see AttnCtx::sm_base.
template <int D, int DV, int NW>
__device__ __forceinline__ void attn_stage_tile(AttnCtx<D, DV, NW> &c, const TilePos &p) {
  using G = AttnGeom<D, DV, NW>;
  const uint32_t last = (uint32_t)min(p.re - 1 - p.k0, kKT - 1);      // last row of the tile that exists
  const char *ktile = reinterpret_cast<const char *>(c.Ks + ((size_t)p.pr * c.r + p.k0) * D);
  const char *vtile = reinterpret_cast<const char *>(c.Vt + (size_t)p.pr * DV * c.r64 + p.k0);
#pragma unroll
  for (int e = 0; e < G::KLOADS; ++e)
    c.stage[e] = *reinterpret_cast<const u32x4 *>(ktile + (min(c.krow + e * G::KROWS_PER_LOAD, last) * (2 * D) + c.kcol));
#pragma unroll
  for (int e = 0; e < G::VLOADS; ++e)
    c.stage[G::KLOADS + e] =
        *reinterpret_cast<const u32x4 *>(vtile + (size_t)e * G::VROWS_PER_LOAD * c.r64 * 2 + c.voff);
  const size_t so = (size_t)p.pr * c.sm_stride + p.k0 * c.sm_tile;
  const float *small = c.sm_base + so, *cap = c.sm_cap + so;
  const uint32_t j = min((uint32_t)c.l, c.sm_tile ? last : 63u);
  c.stage_small = fminf(small[j], cap[j]);
  if constexpr (G::CW == 128) c.stage_small2 = fminf(small[c.sm_tile ? j : j + 64], cap[c.sm_tile ? j : j + 64]);
}

// Stores the staged tile into LDS buffer `wr`: piece e of wave wv is bytes (e NW + wv) 1024 .. + 1023 of the key
// (then value) tile, 16 per lane.
template <int D, int DV, int NW>
__device__ __forceinline__ void attn_store_tile(const AttnCtx<D, DV, NW> &c, char *__restrict__ wr) {
  using G = AttnGeom<D, DV, NW>;
#pragma unroll
  for (int e = 0; e < G::KLOADS; ++e)
    *reinterpret_cast<u32x4 *>(wr + G::OFF_K + e * (G::KROWS_PER_LOAD * G::KROWB) + c.kst) = c.stage[e];
#pragma unroll
  for (int e = 0; e < G::VLOADS; ++e)
    *reinterpret_cast<u32x4 *>(wr + G::OFF_V + e * (G::VROWS_PER_LOAD * G::VROWB) + c.vst) = c.stage[G::KLOADS + e];
  reinterpret_cast<float *>(wr + c.sm_dst)[c.l] = c.stage_small;
  if constexpr (G::CW == 128) reinterpret_cast<float *>(wr + c.sm_dst2)[c.l] = c.stage_small2;
}

template <int D, int DV, int NW>
__device__ __forceinline__ void attn_load_q(AttnCtx<D, DV, NW> &c, int item) {
  const int bh = item / c.qtiles;
  const int64_t q0 = (int64_t)(item % c.qtiles) * (NW * 32) + c.wv * 32;
  const int64_t row = q0 + c.c32 < c.m ? q0 + c.c32 : c.m - 1;
  const uint4 *src = reinterpret_cast<const uint4 *>(c.Q + ((size_t)bh * c.m + row) * D + 8 * c.g);
#pragma unroll
  for (int kb = 0; kb < D / 16; ++kb) {
    const uint4 v = src[2 * kb];
    c.qf[kb] = *reinterpret_cast<const bf16x8 *>(&v);
  }
}

// One 64-key tile of one item: reads LDS buffer `rd` (tile c.cur); first stores the staged tile c.nxt into `wr`
// (free since the barrier that ended the previous tile) and starts the loads of the tile after it.
// Returns false after the last tile of the workgroup's last item.
template <int D, int DV, int NW>
__device__ __forceinline__ bool attn_tile(AttnCtx<D, DV, NW> &c, const char *__restrict__ rd, char *__restrict__ wr,
                                          char *__restrict__ ob) {
  using G = AttnGeom<D, DV, NW>;
  const char *lkr = rd + G::OFF_K + c.kop;                    // this lane's operand row of the first 32 keys, piece g
  const char *lvr = rd + G::OFF_V + c.vop;                    // ... of the first 32 value columns
  const float *lwr = reinterpret_cast<const float *>(rd + G::OFF_W) + 8 * c.g;   // weights of keys 8 g ..
  const int g = c.g, c32 = c.c32;
  const bool last_tile = c.cur.k0 + kKT >= c.cur.re;         // then c.nxt is tile 0 of the workgroup's next item
  const bool more = c.nxt.item < c.total_items;
  attn_store_tile<D, DV, NW>(c, wr);
  // Past the end of the workgroup's list this is a valid tile again (never used), so every tile does the same.
  const TilePos fut = attn_advance(c, c.nxt);
  attn_stage_tile<D, DV, NW>(c, fut);
  // ---- S^T = K Q^T for the two 32-key halves -----------------------------------------------------------
  floatx16 st[2];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int v = 0; v < 16; ++v) st[mt][v] = 0.0f;
  // The K operands are requested two feature blocks (four MFMAs) ahead of their use, through a ring of three
  // operand pairs; the sched_group_barrier sequence below makes the compiler keep that order (left alone it
  // requests each pair right before the MFMAs that need it and then waits out the LDS latency eight times).
  constexpr int KB = D / 16;
  auto k_operand = [&](int kb, int mt) {
    return *reinterpret_cast<const bf16x8 *>(lkr + 32 * mt * G::KROWB + 32 * kb);
  };
  bf16x8 ka[3][2];
#pragma unroll
  for (int kb = 0; kb < 2 && kb < KB; ++kb)
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) ka[kb][mt] = k_operand(kb, mt);
#pragma unroll
  for (int kb = 0; kb < KB; ++kb) {
    if (kb + 2 < KB) {
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) ka[(kb + 2) % 3][mt] = k_operand(kb + 2, mt);
    }
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
      st[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kb % 3][mt], c.qf[kb], st[mt], 0, 0, 0);
  }
  __builtin_amdgcn_sched_group_barrier(kSchedDsRead, 4, 0);
#pragma unroll
  for (int kb = 0; kb + 2 < KB; ++kb) {
    __builtin_amdgcn_sched_group_barrier(kSchedMfma, 2, 0);
    __builtin_amdgcn_sched_group_barrier(kSchedDsRead, 2, 0);
  }
  __builtin_amdgcn_sched_group_barrier(kSchedMfma, 4, 0);
  // The Q fragments are dead after the last score product of an item: the next item's are loaded into the same
  // registers now and arrive during the softmax, value product and epilogue of this tile.
  if (last_tile && more) {
    attn_load_q<D, DV, NW>(c, c.nxt.item);
    c.nvsc = c.vscale[c.nxt.pr];
  }
  if (c.cur.k0 + kKT > c.cur.re) {                           // ragged last tile: mask the missing keys
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (c.cur.k0 + 32 * mt + 16 * (v / 8) + 8 * g + 4 * ((v / 4) % 2) + (v % 4) >= c.cur.re) st[mt][v] = -INFINITY;
  }
  // ---- row maximum of the raw scores; move the reference only if it is more than the slack behind ------------
  float mx = st[0][0];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt)
#pragma unroll
    for (int v = 0; v < 16; ++v) mx = fmaxf(mx, st[mt][v]);
  mx = pair_max(mx) * c.scale_log2;
  const bool jump = mx > c.mref + kRescaleSlack;
  if (c.cur.k0 == 0) {
    c.mref = mx;                                             // first tile of an item: sums and accumulators are zero
  } else if (__builtin_amdgcn_ballot_w64(jump) != 0) {
    const float alpha = jump ? __builtin_amdgcn_exp2f(c.mref - mx) : 1.0f;
    c.mref = jump ? mx : c.mref;
    c.den *= alpha;
#pragma unroll
    for (int i = 0; i < DV / 32; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) c.acc[i][v] *= alpha;
  }
  // ---- P = exp2(S c - mref), normaliser, fp16 operand (packed conversion, rounds toward zero: the common
  // relative shortfall of the terms is far below the output rounding, their scatter is that of round-to-nearest) ----
  const float nm = -c.mref;
  float dl = 0.0f;
  f16x8 pf[4];
#pragma unroll
  for (int mt = 0; mt < 2; ++mt) {
    floatx16 p;
#pragma unroll
    for (int v = 0; v < 16; ++v) p[v] = __builtin_amdgcn_exp2f(fmaf(st[mt][v], c.scale_log2, nm));
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const float4 wv4 = *reinterpret_cast<const float4 *>(&lwr[32 * mt + 16 * (q / 2) + 4 * (q % 2)]);
      dl = fmaf(p[4 * q + 0], wv4.x, dl);
      dl = fmaf(p[4 * q + 1], wv4.y, dl);
      dl = fmaf(p[4 * q + 2], wv4.z, dl);
      dl = fmaf(p[4 * q + 3], wv4.w, dl);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const auto h0 = __builtin_amdgcn_cvt_pkrtz(p[8 * h + 0], p[8 * h + 1]);
      const auto h1 = __builtin_amdgcn_cvt_pkrtz(p[8 * h + 2], p[8 * h + 3]);
      const auto h2 = __builtin_amdgcn_cvt_pkrtz(p[8 * h + 4], p[8 * h + 5]);
      const auto h3 = __builtin_amdgcn_cvt_pkrtz(p[8 * h + 6], p[8 * h + 7]);
      const uint4 hb = make_uint4(*reinterpret_cast<const uint32_t *>(&h0), *reinterpret_cast<const uint32_t *>(&h1),
                                  *reinterpret_cast<const uint32_t *>(&h2), *reinterpret_cast<const uint32_t *>(&h3));
      pf[2 * mt + h] = *reinterpret_cast<const f16x8 *>(&hb);
    }
  }
  c.den += dl;
  // ---- O^T += V_S^T P^T: A operand = keys 16kb + 8g + 0..7 of value column c32, one 16-byte piece ---------------
#pragma unroll
  for (int kb = 0; kb < 4; ++kb) {
#pragma unroll
    for (int i = 0; i < DV / 32; ++i) {
      const f16x8 av = *reinterpret_cast<const f16x8 *>(lvr + 32 * i * G::VROWB + 32 * kb);
      c.acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(av, pf[kb], c.acc[i], 0, 0, 0);
    }
  }
  if (last_tile) {
    // ---- epilogue of the item: guard, divide, clip, store; then start the next item --------------------------------
    const float dn = pair_sum(c.den);
    const bool ok = dn > 0.0f;
    const float inv = ok ? c.vsc / dn : 0.0f;               // v_t holds V_S^T / v_scale
    // The accumulators hold a query's row in 8-byte bits spread over (i, q); stored from there, every store would
    // touch 32 rows with 8 bytes each.  So the converted values go through this wave's corner of LDS, 64 columns at
    // a time, and leave as whole 128-byte lines (16 bytes per lane, eight rows per store).  No barrier: only this
    // wave touches its corner, and a wave's LDS operations complete in order.
    const int bh = c.cur.item / c.qtiles;
    const int64_t q0 = (int64_t)(c.cur.item % c.qtiles) * (NW * 32) + c.wv * 32;
    bf16_t *obase = c.out + ((size_t)bh * c.m + q0) * DV;
    const float *clip = reinterpret_cast<const float *>(rd + G::OFF_C);
    char *mine = ob + c.wv * (32 * G::OROWB);
#pragma unroll
    for (int h = 0; h < DV / 64; ++h) {
#pragma unroll
      for (int ii = 0; ii < 2; ++ii)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int i = 2 * h + ii, col = 32 * i + 8 * q + 4 * g;
          const float4 lo = *reinterpret_cast<const float4 *>(&clip[col]);
          const float4 hi = *reinterpret_cast<const float4 *>(&clip[DV + col]);
          // inv = 0 where the guard fails (the accumulators are finite: P <= 2^8, |v_t| < 2^15).  The lower bounds
          // in LDS are min(v_min, v_max), so the median of three is min(max(o, v_min), v_max) for any bounds.
          floatx4 o = {c.acc[i][4 * q + 0] * inv, c.acc[i][4 * q + 1] * inv, c.acc[i][4 * q + 2] * inv,
                       c.acc[i][4 * q + 3] * inv};
          o[0] = __builtin_amdgcn_fmed3f(o[0], lo.x, hi.x);
          o[1] = __builtin_amdgcn_fmed3f(o[1], lo.y, hi.y);
          o[2] = __builtin_amdgcn_fmed3f(o[2], lo.z, hi.z);
          o[3] = __builtin_amdgcn_fmed3f(o[3], lo.w, hi.w);
          const bf16x4 ob4 = __builtin_convertvector(o, bf16x4);
          *reinterpret_cast<uint2 *>(mine + c32 * G::OROWB + (col - 64 * h) * 2) = *reinterpret_cast<const uint2 *>(&ob4);
        }
#pragma unroll
      for (int j = 0; j < 4; ++j) {                            // 32 rows x 128 bytes = 256 pieces of 16
        const int idx = j * 64 + c.l, row = idx / 8, piece = idx % 8;
        const uint4 v = *reinterpret_cast<const uint4 *>(mine + row * G::OROWB + piece * 16);
        if (q0 + row < c.m) *reinterpret_cast<uint4 *>(obase + (size_t)row * DV + 64 * h + piece * 8) = v;
      }
    }
    if (!more) return false;
#pragma unroll
    for (int i = 0; i < DV / 32; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) c.acc[i][v] = 0.0f;
    c.mref = -INFINITY;
    c.den = 0.0f;
    c.vsc = c.nvsc;
  }
  // The stores into `wr` have completed (lgkmcnt(0); 0xC07F leaves the other counters alone) and every LDS read of
  // this tile has been consumed by the MFMAs and sums above, so after the barrier `wr` may be read and `rd`
  // overwritten.  A bare s_barrier on purpose: __syncthreads() would also wait for the loads in flight.
  __builtin_amdgcn_s_waitcnt(0xC07F);
  __builtin_amdgcn_s_barrier();
  c.cur = c.nxt;
  c.nxt = fut;
  return true;
}

template <int D, int DV, int NW>
__global__ __launch_bounds__(NW * 64, 1) void k_wtd_attn_mfma2(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ Ks, const uint16_t *__restrict__ Vt,
    const float *__restrict__ vscale, const float *__restrict__ w, const float *__restrict__ vmin,
    const float *__restrict__ vmax, const int32_t *__restrict__ r_eff, bf16_t *__restrict__ out, int64_t m, int r,
    int r64, int q_heads, int group, int qtiles, int total_items, float scale_log2) {
  using G = AttnGeom<D, DV, NW>;
  __shared__ __attribute__((aligned(16))) char buf0[G::BYTES];
  __shared__ __attribute__((aligned(16))) char buf1[G::BYTES];
  __shared__ __attribute__((aligned(16))) char obuf[G::OBYTES];     // output staging, see the epilogue in attn_tile

  AttnCtx<D, DV, NW> c;
  c.Q = Q; c.Ks = Ks; c.Vt = Vt; c.vscale = vscale; c.w = w; c.vmin = vmin; c.vmax = vmax; c.r_eff = r_eff; c.out = out;
  c.m = m; c.r = r; c.r64 = r64; c.q_heads = q_heads; c.group = group; c.kv_heads = q_heads / group;
  c.qtiles = qtiles; c.total_items = total_items; c.stride = (int)gridDim.x; c.scale_log2 = scale_log2;
  const int t = threadIdx.x;
  c.wv = __builtin_amdgcn_readfirstlane(t / kWave);          // wave-uniform: keep it in a scalar register
  c.l = t % kWave; c.g = c.l / 32; c.c32 = c.l % 32;
  c.kop = c.c32 * G::KROWB + c.g * 16;
  c.vop = c.c32 * G::VROWB + c.g * 16;
  {                                           // piece wv 64 + l of the key tile: piece `slot` of LDS row `row`
    const int idx = c.wv * 64 + c.l, row = idx / G::KPPR, slot = idx % G::KPPR;
    // LDS row `row` holds key pi(row), see attn_tile; pi commutes with steps of KROWS_PER_LOAD rows
    static_assert(G::KROWS_PER_LOAD % 16 == 0, "the row permutation acts on bits 2 and 3");
    c.krow = (row & ~12) | ((row & 4) << 1) | ((row & 8) >> 1);
    c.kcol = slot * 16;
    c.kst = row * G::KROWB + slot * 16;
  }
  {
    const int idx = c.wv * 64 + c.l, row = idx / G::VPPR, slot = idx % G::VPPR;
    c.voff = (uint32_t)(row * r64 + slot * 8) * 2;
    c.vst = row * G::VROWB + slot * 16;
  }

  static_assert(DV % G::CW == 0, "a wave's clip entries lie in v_min or in v_max, not across");
  if (c.wv >= 1 && c.wv <= G::CLOADS) {
    const int q = c.wv - 1;                                   // entries CW q .. CW q + CW - 1 of v_min | v_max
    c.sm_base = q < DV / G::CW ? vmin + G::CW * q : vmax + (G::CW * q - DV);
    c.sm_cap = q < DV / G::CW ? vmax + G::CW * q : c.sm_base;
    c.sm_stride = DV; c.sm_tile = 0; c.sm_dst = G::OFF_C + 4 * G::CW * q; c.sm_dst2 = c.sm_dst + 256;
  } else {
    c.sm_base = c.sm_cap = w;
    c.sm_stride = r; c.sm_tile = 1; c.sm_dst = c.wv == 0 ? G::OFF_W : G::OFF_SPARE; c.sm_dst2 = G::OFF_SPARE + 256;
  }
  // An item is one (batch*head, query tile) pair; this workgroup takes items blockIdx.x, + gridDim.x, ...
  c.cur.item = blockIdx.x;
  if (c.cur.item >= total_items) return;
  c.cur.pr = attn_item_pr(c, c.cur.item);
  c.cur.re = attn_item_re(c, c.cur.pr);
  c.cur.k0 = 0;
  c.nxt = attn_advance(c, c.cur);
  attn_stage_tile<D, DV, NW>(c, c.cur);
  attn_store_tile<D, DV, NW>(c, buf0);
  attn_stage_tile<D, DV, NW>(c, c.nxt);
  attn_load_q<D, DV, NW>(c, c.cur.item);
#pragma unroll
  for (int i = 0; i < DV / 32; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) c.acc[i][v] = 0.0f;
  c.mref = -INFINITY;
  c.den = 0.0f;
  c.vsc = c.nvsc = vscale[c.cur.pr];
  __syncthreads();                         // tile 0 is in buf0
  while (attn_tile<D, DV, NW>(c, buf0, buf1, obuf) && attn_tile<D, DV, NW>(c, buf1, buf0, obuf)) {
  }
}

// --------------------------------------------------------------------------------------------
// Decode shape: few queries per head (new tokens against a stored coreset).  The kernel above would run one
// workgroup per head through all r keys in sequence, seven of its eight waves idle at m = 1.  Here the query heads
// that share a kv head are packed into one block of 32 rows (row = head-in-group * m + query), and the key tiles of
// the coreset are dealt out to the eight waves of the workgroup, which combine their partial (reference, normaliser,
// accumulators) through LDS at the end.  No tile is used by two waves, so nothing is staged in LDS: each lane loads
// its MFMA operands straight from memory -- the key row pi(l % 32) of the tile (same row order as in the kernel
// above) and the piece of v_t for its value column.  Same arithmetic per tile as above (bf16 scores, fp16 value
// product, fp32 everything else); the sum over the tiles is taken in a different order.
// --------------------------------------------------------------------------------------------
constexpr int kDecWaves = 8;
constexpr int kDecodeRows = 256;                               // packed rows per kv head up to which the decode kernel is used

template <int D, int DV>
__global__ __launch_bounds__(kDecWaves * 64, 1) void k_wtd_attn_decode(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ Ks, const uint16_t *__restrict__ Vt,
    const float *__restrict__ vscale, const float *__restrict__ w, const float *__restrict__ vmin,
    const float *__restrict__ vmax, const int32_t *__restrict__ r_eff, bf16_t *__restrict__ out, int m, int r, int r64,
    int q_heads, int group, float scale_log2) {
  __shared__ float s_ref[kDecWaves][64], s_den[kDecWaves][64];
  __shared__ float s_acc[kDecWaves][DV / 32 * 16][64];         // [wave][accumulator register][lane]
  const int t = threadIdx.x, wv = __builtin_amdgcn_readfirstlane(t / kWave), l = t % kWave, g = l / 32, c32 = l % 32;
  const int pr = blockIdx.y, kv_heads = q_heads / group, b = pr / kv_heads, kvh = pr % kv_heads;
  const int re = r_eff ? max(min(r_eff[pr], r), 1) : r;
  const int rows = group * m;                                  // packed rows of this kv head
  const int row = min((int)blockIdx.x * 32 + c32, rows - 1);   // this lane's query (clamped duplicates are not stored)
  const int hq = kvh * group + row / m, qi = row % m;
  const bf16_t *qrow = Q + (((size_t)b * q_heads + hq) * m + qi) * D;
  bf16x8 qf[D / 16];
#pragma unroll
  for (int kb = 0; kb < D / 16; ++kb) {
    const uint4 v = *reinterpret_cast<const uint4 *>(qrow + 16 * kb + 8 * g);
    qf[kb] = *reinterpret_cast<const bf16x8 *>(&v);
  }
  floatx16 acc[DV / 32];
#pragma unroll
  for (int i = 0; i < DV / 32; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
  float mref = -INFINITY, den = 0.0f;
  const bf16_t *Kp = Ks + (size_t)pr * r * D;
  const uint16_t *Vp = Vt + (size_t)pr * DV * r64;
  const float *wp = w + (size_t)pr * r;
  const int pi = (c32 & ~12) | ((c32 & 4) << 1) | ((c32 & 8) >> 1);   // row order of a key tile, see above

  for (int k0 = wv * kKT; k0 < re; k0 += kDecWaves * kKT) {
    // ---- S^T = K Q^T for the two 32-key halves, operands from memory --------------------------------------
    floatx16 st[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
      for (int v = 0; v < 16; ++v) st[mt][v] = 0.0f;
      const bf16_t *krow = Kp + (size_t)min(k0 + 32 * mt + pi, re - 1) * D + 8 * g;
#pragma unroll
      for (int kb = 0; kb < D / 16; ++kb) {
        const uint4 kv4 = *reinterpret_cast<const uint4 *>(krow + 16 * kb);
        st[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(&kv4), qf[kb], st[mt], 0, 0, 0);
      }
    }
    if (k0 + kKT > re) {                                       // ragged last tile: mask the missing keys
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (k0 + 32 * mt + 16 * (v / 8) + 8 * g + 4 * ((v / 4) % 2) + (v % 4) >= re) st[mt][v] = -INFINITY;
    }
    float mx = st[0][0];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, st[mt][v]);
    mx = pair_max(mx) * scale_log2;                            // finite: key k0 exists
    if (mx > mref) {                                           // true running maximum: a wave sees few tiles
      const float alpha = __builtin_amdgcn_exp2f(mref - mx);   // 0 on the first tile
      mref = mx;
      den *= alpha;
#pragma unroll
      for (int i = 0; i < DV / 32; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] *= alpha;
    }
    const float nm = -mref;
    float dl = 0.0f;
    f16x8 pf[4];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      floatx16 p;
#pragma unroll
      for (int v = 0; v < 16; ++v) p[v] = __builtin_amdgcn_exp2f(fmaf(st[mt][v], scale_log2, nm));
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int key = k0 + 32 * mt + 16 * (q / 2) + 8 * g + 4 * (q % 2);
#pragma unroll
        for (int e = 0; e < 4; ++e) dl = fmaf(p[4 * q + e], wp[min(key + e, re - 1)], dl);   // p is 0 past re
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const auto h0 = __builtin_amdgcn_cvt_pkrtz(p[8 * h + 0], p[8 * h + 1]);
        const auto h1 = __builtin_amdgcn_cvt_pkrtz(p[8 * h + 2], p[8 * h + 3]);
        const auto h2 = __builtin_amdgcn_cvt_pkrtz(p[8 * h + 4], p[8 * h + 5]);
        const auto h3 = __builtin_amdgcn_cvt_pkrtz(p[8 * h + 6], p[8 * h + 7]);
        const uint4 hb = make_uint4(*reinterpret_cast<const uint32_t *>(&h0), *reinterpret_cast<const uint32_t *>(&h1),
                                    *reinterpret_cast<const uint32_t *>(&h2), *reinterpret_cast<const uint32_t *>(&h3));
        pf[2 * mt + h] = *reinterpret_cast<const f16x8 *>(&hb);
      }
    }
    den += dl;
    // ---- O^T += V_S^T P^T: A operand = keys k0 + 16 kb + 8 g + 0..7 of value column 32 i + c32 (v_t is zero padded) ----
#pragma unroll
    for (int kb = 0; kb < 4; ++kb)
#pragma unroll
      for (int i = 0; i < DV / 32; ++i) {
        const uint4 vv = *reinterpret_cast<const uint4 *>(Vp + (size_t)(32 * i + c32) * r64 + k0 + 16 * kb + 8 * g);
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(*reinterpret_cast<const f16x8 *>(&vv), pf[kb], acc[i], 0, 0, 0);
      }
  }

  // ---- combine the waves' partial results: common reference = the largest one --------------------------------------
  s_ref[wv][l] = mref;
  __syncthreads();
  float mall = s_ref[0][l];
#pragma unroll
  for (int k = 1; k < kDecWaves; ++k) mall = fmaxf(mall, s_ref[k][l]);
  const float sc = __builtin_amdgcn_exp2f(mref - mall);        // wave 0 always has a tile, so mall is finite; 0 for idle waves
  s_den[wv][l] = den * sc;
#pragma unroll
  for (int i = 0; i < DV / 32; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s_acc[wv][16 * i + v][l] = acc[i][v] * sc;
  __syncthreads();
  float dsum = 0.0f;
#pragma unroll
  for (int k = 0; k < kDecWaves; ++k) dsum += s_den[k][l];
  const float dn = pair_sum(dsum);
  const bool ok = dn > 0.0f;
  const float inv = ok ? vscale[pr] / dn : 0.0f;               // v_t holds V_S^T / v_scale
  // wave wv finishes accumulator registers [R wv, R (wv + 1)): block i = reg / 16, v = reg % 16 <-> column
  // 32 i + 8 (v / 4) + 4 g + v % 4, i.e. four registers = four consecutive columns
  constexpr int R = DV / 32 * 16 / kDecWaves;                 // 8 at dv = 128, 4 at dv = 64
  static_assert(R % 4 == 0, "whole groups of four columns per wave");
  if ((int)blockIdx.x * 32 + c32 < rows) {
    bf16_t *orow = out + (((size_t)b * q_heads + hq) * m + qi) * DV;
#pragma unroll
    for (int q4 = 0; q4 < R / 4; ++q4) {
      const int reg = R * wv + 4 * q4, i = reg / 16, v = reg % 16, col = 32 * i + 8 * (v / 4) + 4 * g;
      floatx4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float a = 0.0f;
#pragma unroll
        for (int k = 0; k < kDecWaves; ++k) a += s_acc[k][reg + e][l];
        a = ok ? a * inv : 0.0f;
        o[e] = fminf(fmaxf(a, vmin[(size_t)pr * DV + col + e]), vmax[(size_t)pr * DV + col + e]);
      }
      const bf16x4 ob = __builtin_convertvector(o, bf16x4);
      *reinterpret_cast<uint2 *>(orow + col) = *reinterpret_cast<const uint2 *>(&ob);
    }
  }
}

template <int D, int DV>
int launch_decode(const Shape &s, const void *Q, const wildcat_coreset *cs, void *out) {
  const int r64 = (s.r + 63) / 64 * 64;
  const int rows = s.group * (int)s.m;
  const dim3 grid((unsigned)((rows + 31) / 32), (unsigned)s.P);
  hipLaunchKernelGGL((k_wtd_attn_decode<D, DV>), grid, dim3(kDecWaves * 64), 0, s.stream, (const bf16_t *)Q,
                     (const bf16_t *)cs->k_s, (const uint16_t *)cs->v_t, cs->v_scale, cs->w, cs->v_min, cs->v_max,
                     cs->r_eff, (bf16_t *)out, (int)s.m, s.r, r64, s.q_heads, s.group,
                     (float)(s.beta * (double)kLog2e));
  return hipGetLastError() == hipSuccess ? WILDCAT_OK : WILDCAT_EHIP;
}

// --------------------------------------------------------------------------------------------
// MFMA kernel for fp32 storage (d, dv multiples of the MFMA tile).  Same transposed arrangement as the bf16 kernel,
// on v_mfma_f32_32x32x2_f32: lane l of the A operand (32 x 2) holds row l % 32, k = l / 32; of the B operand (2 x 32)
// column l % 32, k = l / 32; D as for the other 32 x 32 shapes.  Everything stays fp32: S^T = K_S Q^T, P = exp2(...)
// in registers, O^T = V_S^T P^T with P straight from the S^T registers as the B operand.  Register v of an S^T tile
// holds key 8 (v / 4) + v % 4 in lanes 0..31 and that key + 4 in lanes 32..63, so step v of the value product
// contracts over exactly these two keys and the A operand is V_S[that key][32 i + l % 32] (a 4-byte LDS read, row
// stride padded by 8 floats so that the two lane halves fall into different banks).  The contraction index of the
// score product is permuted likewise: step 4 t + u of lane half g uses feature 8 t + 4 g + u, so a lane reads its
// key's features 8 t + 4 g .. + 3 with one 16-byte LDS read (row stride padded by 4 floats: every 16-byte bank
// group is hit by four lanes, which is the best 64 lanes x 16 bytes can do) and holds the matching half of its
// query row in registers.  Workgroup = NWF waves x 32 queries; 32-key tiles of K_S, V_S and w through LDS.
// --------------------------------------------------------------------------------------------
constexpr int kFT = 32;                                       // keys per tile

template <int D, int DV, int NWF>
__global__ __launch_bounds__(NWF * 64) void k_wtd_attn_mfma_f32(
    const float *__restrict__ Q, const float *__restrict__ Ks, const float *__restrict__ Vs,
    const float *__restrict__ w, const float *__restrict__ vmin, const float *__restrict__ vmax,
    const int32_t *__restrict__ r_eff, float *__restrict__ out, int64_t m, int r, int q_heads, int group,
    float scale_log2) {
  constexpr int KROW = D + 4, VROW = DV + 8;                  // padded LDS row strides (floats)
  __shared__ __attribute__((aligned(16))) float lk[kFT * KROW];
  __shared__ __attribute__((aligned(16))) float lv[kFT * VROW];
  __shared__ float lw[kFT];
  const int t = threadIdx.x, wv = t / kWave, l = t % kWave, g = l / 32, c32 = l % 32;
  const int bh = blockIdx.y, b = bh / q_heads, hq = bh % q_heads;
  const int pr = b * (q_heads / group) + hq / group;
  const int re = r_eff ? max(min(r_eff[pr], r), 1) : r;
  const int64_t q0 = (int64_t)blockIdx.x * (NWF * 32) + wv * 32;
  const int64_t qrow = q0 + c32 < m ? q0 + c32 : m - 1;

  // this lane's half of its query row: features 8 t + 4 g + u
  float qf[D / 2];
  {
    const float4 *src = reinterpret_cast<const float4 *>(Q + ((size_t)bh * m + qrow) * D + 4 * g);
#pragma unroll
    for (int tt = 0; tt < D / 8; ++tt) {
      const float4 v = src[2 * tt];
      qf[4 * tt + 0] = v.x; qf[4 * tt + 1] = v.y; qf[4 * tt + 2] = v.z; qf[4 * tt + 3] = v.w;
    }
  }
  floatx16 acc[DV / 32];
#pragma unroll
  for (int i = 0; i < DV / 32; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
  float mrun = -INFINITY, den = 0.0f;
  const float *Kp = Ks + (size_t)pr * r * D, *Vp = Vs + (size_t)pr * r * DV, *wp = w + (size_t)pr * r;

  // A tile travels memory -> registers -> LDS.  Where the registers allow it (PREFETCH) the loads of tile t+1 are
  // issued right after tile t has been stored to LDS, so they fly during the MFMAs of tile t.
  constexpr int NT = NWF * 64, KR = kFT * (D / 4) / NT, VR = kFT * (DV / 4) / NT;
  static_assert(KR * NT == kFT * (D / 4) && VR * NT == kFT * (DV / 4), "tiles must split evenly");
  constexpr bool PREFETCH = DV <= 128 || NWF >= 4;          // (staging registers per thread shrink with the workgroup)
  float4 kreg[KR], vreg[VR];
  float wreg = 0.0f;
  auto fetch = [&](int k0) {
#pragma unroll
    for (int q = 0; q < KR; ++q) {
      const int e = t + q * NT, kk = e / (D / 4), j = e % (D / 4);
      kreg[q] = k0 + kk < re ? *reinterpret_cast<const float4 *>(Kp + (size_t)(k0 + kk) * D + 4 * j)
                             : make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int q = 0; q < VR; ++q) {
      const int e = t + q * NT, kk = e / (DV / 4), j = e % (DV / 4);
      vreg[q] = k0 + kk < re ? *reinterpret_cast<const float4 *>(Vp + (size_t)(k0 + kk) * DV + 4 * j)
                             : make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (t < kFT) wreg = k0 + t < re ? wp[k0 + t] : 0.0f;
  };
  if (PREFETCH) fetch(0);

  for (int k0 = 0; k0 < re; k0 += kFT) {
    if (!PREFETCH) fetch(k0);
    __syncthreads();                                          // the previous tile has been read
#pragma unroll
    for (int q = 0; q < KR; ++q) {
      const int e = t + q * NT, kk = e / (D / 4), j = e % (D / 4);
      *reinterpret_cast<float4 *>(&lk[kk * KROW + 4 * j]) = kreg[q];
    }
#pragma unroll
    for (int q = 0; q < VR; ++q) {
      const int e = t + q * NT, kk = e / (DV / 4), j = e % (DV / 4);
      *reinterpret_cast<float4 *>(&lv[kk * VROW + 4 * j]) = vreg[q];
    }
    if (t < kFT) lw[t] = wreg;
    __syncthreads();
    if (PREFETCH && k0 + kFT < re) fetch(k0 + kFT);
    // ---- S^T = K Q^T --------------------------------------------------------------------------------------
    floatx16 st;
#pragma unroll
    for (int v = 0; v < 16; ++v) st[v] = 0.0f;
#pragma unroll
    for (int tt = 0; tt < D / 8; ++tt) {
      const float4 a = *reinterpret_cast<const float4 *>(&lk[c32 * KROW + 8 * tt + 4 * g]);
      st = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, qf[4 * tt + 0], st, 0, 0, 0);
      st = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, qf[4 * tt + 1], st, 0, 0, 0);
      st = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, qf[4 * tt + 2], st, 0, 0, 0);
      st = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, qf[4 * tt + 3], st, 0, 0, 0);
    }
    // register v <-> key k0 + 8 (v / 4) + 4 g + v % 4
    float mx = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      st[v] = k0 + 8 * (v / 4) + 4 * g + (v % 4) < re ? st[v] * scale_log2 : -INFINITY;
      mx = fmaxf(mx, st[v]);
    }
    mx = pair_max(mx);
    const float mnew = fmaxf(mrun, mx);                       // finite: key k0 exists
    const float alpha = __builtin_amdgcn_exp2f(mrun - mnew);
    mrun = mnew;
    float dl = 0.0f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      st[v] = __builtin_amdgcn_exp2f(st[v] - mnew);
      dl = fmaf(st[v], lw[8 * (v / 4) + 4 * g + (v % 4)], dl);
    }
    den = den * alpha + dl;
    // ---- O^T = alpha O^T + V^T P^T ---------------------------------------------------------------------------
#pragma unroll
    for (int i = 0; i < DV / 32; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][v] *= alpha;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float *vrow = &lv[(8 * (v / 4) + 4 * g + (v % 4)) * VROW + c32];
#pragma unroll
      for (int i = 0; i < DV / 32; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(vrow[32 * i], st[v], acc[i], 0, 0, 0);
    }
  }
  // ---- epilogue: guard, divide, clip, store (register v of block i <-> column 32 i + 8 (v / 4) + 4 g + v % 4) ----------
  const float dn = pair_sum(den);
  const bool ok = dn > 0.0f;
  const float inv = ok ? 1.0f / dn : 0.0f;
  if (q0 + c32 < m) {
    float *orow = out + ((size_t)bh * m + q0 + c32) * DV;
#pragma unroll
    for (int i = 0; i < DV / 32; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = 32 * i + 8 * q + 4 * g;
        const float4 lo = *reinterpret_cast<const float4 *>(vmin + (size_t)pr * DV + col);
        const float4 hi = *reinterpret_cast<const float4 *>(vmax + (size_t)pr * DV + col);
        float4 o = make_float4(acc[i][4 * q + 0] * inv, acc[i][4 * q + 1] * inv, acc[i][4 * q + 2] * inv,
                               acc[i][4 * q + 3] * inv);
        if (!ok) o = make_float4(0.f, 0.f, 0.f, 0.f);
        o.x = fminf(fmaxf(o.x, lo.x), hi.x);
        o.y = fminf(fmaxf(o.y, lo.y), hi.y);
        o.z = fminf(fmaxf(o.z, lo.z), hi.z);
        o.w = fminf(fmaxf(o.w, lo.w), hi.w);
        *reinterpret_cast<float4 *>(orow + col) = o;
      }
  }
}


// Few queries in all (the image-model layer shapes: a few thousand queries per head, a handful of heads): 32 queries
// per wavefront leave most SIMDs without a wave and the others with one, which waits out every load and every MFMA
// chain.  Here a workgroup still owns one block of 32 queries, but its NS wavefronts share out the key tiles of the
// coreset (tile wv, wv + NS, ...), each with its own running reference, normaliser and accumulators, and combine them
// through LDS at the end -- as the bf16 decode kernel does.  No tile is used by two waves of a workgroup, so nothing
// is staged in LDS: a lane reads its MFMA operands straight from memory (the coreset is small and stays in the L2),
// in the same arrangement as the kernel above.  Same arithmetic per tile; the tiles are summed in another order.
// grid (ceil(m / 32), batch * q_heads); dynamic LDS NS x (DV / 2) x 64 floats.
template <int D, int DV, int NS>
__global__ __launch_bounds__(NS * 64, 2) void k_wtd_attn_f32_split(
    const float *__restrict__ Q, const float *__restrict__ Ks, const float *__restrict__ Vs,
    const float *__restrict__ w, const float *__restrict__ vmin, const float *__restrict__ vmax,
    const int32_t *__restrict__ r_eff, float *__restrict__ out, int64_t m, int r, int q_heads, int group,
    float scale_log2) {
  constexpr int NR = DV / 32 * 16;                            // accumulator registers per lane
  static_assert(NR % (4 * NS) == 0, "every wave finishes whole groups of four columns");
  __shared__ float s_ref[NS][64], s_den[NS][64];
  extern __shared__ float s_acc[];                            // [NS][NR][64]
  const int t = threadIdx.x, wv = __builtin_amdgcn_readfirstlane(t / kWave), l = t % kWave, g = l / 32, c32 = l % 32;
  const int bh = blockIdx.y, b = bh / q_heads, hq = bh % q_heads;
  const int pr = b * (q_heads / group) + hq / group;
  const int re = r_eff ? max(min(r_eff[pr], r), 1) : r;
  const int64_t q0 = (int64_t)blockIdx.x * 32;
  const int64_t qrow = q0 + c32 < m ? q0 + c32 : m - 1;
  float qf[D / 2];                                            // this lane's half of its query row: features 8 t + 4 g + u
  {
    const float4 *src = reinterpret_cast<const float4 *>(Q + ((size_t)bh * m + qrow) * D + 4 * g);
#pragma unroll
    for (int tt = 0; tt < D / 8; ++tt) {
      const float4 v = src[2 * tt];
      qf[4 * tt + 0] = v.x; qf[4 * tt + 1] = v.y; qf[4 * tt + 2] = v.z; qf[4 * tt + 3] = v.w;
    }
  }
  floatx16 acc[DV / 32];
#pragma unroll
  for (int i = 0; i < DV / 32; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
  float mrun = -INFINITY, den = 0.0f;
  const float *Kp = Ks + (size_t)pr * r * D, *Vp = Vs + (size_t)pr * r * DV, *wp = w + (size_t)pr * r;

  // Where the registers allow it (PF: d = d_v = 64) a wave keeps its loads a tile ahead of its MFMAs: the values and
  // weights of its next tile are requested before the current tile's score product, the keys of the next tile right
  // after it, so after the first tile nothing waits for memory (the scheduling barriers keep the requests there).
  constexpr bool PF = D <= 64 && DV <= 64;
  auto load_keys = [&](int k0, float4 (&ka)[D / 8]) {
    const float *krow = Kp + (size_t)min(k0 + c32, re - 1) * D + 4 * g;
#pragma unroll
    for (int tt = 0; tt < D / 8; ++tt) ka[tt] = *reinterpret_cast<const float4 *>(krow + 8 * tt);
  };
  auto load_values = [&](int k0, float (&vv)[PF ? 16 : 1][PF ? DV / 32 : 1], float (&ww)[16]) {
    if constexpr (PF) {
      if (k0 + kFT <= re) {
        // a whole tile: one pointer per lane and compile-time offsets from it (k0 is the same in every lane)
        const float *vl = Vp + (size_t)k0 * DV + (4 * g * DV + c32), *wl = wp + k0 + 4 * g;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          ww[v] = wl[8 * (v / 4) + (v % 4)];
#pragma unroll
          for (int i = 0; i < DV / 32; ++i) vv[v][i] = vl[(8 * (v / 4) + (v % 4)) * DV + 32 * i];
        }
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const unsigned key = (unsigned)min(k0 + 8 * (v / 4) + 4 * g + (v % 4), re - 1);
          ww[v] = wp[key];
#pragma unroll
          for (int i = 0; i < DV / 32; ++i) vv[v][i] = Vp[key * (unsigned)DV + (unsigned)(c32 + 32 * i)];
        }
      }
    }
  };
  float4 ka[D / 8];
  float vn[PF ? 16 : 1][PF ? DV / 32 : 1], wn[16];
  if (PF && wv * kFT < re) {
    load_keys(wv * kFT, ka);
    load_values(wv * kFT, vn, wn);
  }
  for (int k0 = wv * kFT; k0 < re; k0 += NS * kFT) {
    float wk[16];
    float va[PF ? 16 : 1][PF ? DV / 32 : 1];
    if constexpr (PF) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        wk[v] = wn[v];
#pragma unroll
        for (int i = 0; i < DV / 32; ++i) va[v][i] = vn[v][i];
      }
      if (k0 + NS * kFT < re) load_values(k0 + NS * kFT, vn, wn);
      __builtin_amdgcn_sched_barrier(0);
    } else {
      load_keys(k0, ka);
    }
    // ---- S^T = K Q^T: A operand = key k0 + c32 (clamped; masked below), features 8 t + 4 g .. + 3 ------------------
    floatx16 st;
#pragma unroll
    for (int v = 0; v < 16; ++v) st[v] = 0.0f;
#pragma unroll
    for (int tt = 0; tt < D / 8; ++tt) {
      const float4 a = ka[tt];
      st = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, qf[4 * tt + 0], st, 0, 0, 0);
      st = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, qf[4 * tt + 1], st, 0, 0, 0);
      st = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, qf[4 * tt + 2], st, 0, 0, 0);
      st = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, qf[4 * tt + 3], st, 0, 0, 0);
    }
    if constexpr (PF) {
      if (k0 + NS * kFT < re) load_keys(k0 + NS * kFT, ka);
      __builtin_amdgcn_sched_barrier(0);
    }
    // register v <-> key k0 + 8 (v / 4) + 4 g + v % 4
    float mx = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int key = k0 + 8 * (v / 4) + 4 * g + (v % 4);
      if constexpr (!PF) wk[v] = wp[min(key, re - 1)];
      st[v] = key < re ? st[v] * scale_log2 : -INFINITY;
      mx = fmaxf(mx, st[v]);
    }
    mx = pair_max(mx);
    const float mnew = fmaxf(mrun, mx);                       // finite: key k0 exists
    const float alpha = __builtin_amdgcn_exp2f(mrun - mnew);
    mrun = mnew;
    float dl = 0.0f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      st[v] = __builtin_amdgcn_exp2f(st[v] - mnew);           // 0 for the masked keys
      dl = fmaf(st[v], wk[v], dl);
    }
    den = den * alpha + dl;
#pragma unroll
    for (int i = 0; i < DV / 32; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][v] *= alpha;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      if constexpr (PF) {
#pragma unroll
        for (int i = 0; i < DV / 32; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(va[v][i], st[v], acc[i], 0, 0, 0);
      } else {
        const float *vrow = Vp + (size_t)min(k0 + 8 * (v / 4) + 4 * g + (v % 4), re - 1) * DV + c32;
#pragma unroll
        for (int i = 0; i < DV / 32; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(vrow[32 * i], st[v], acc[i], 0, 0, 0);
      }
    }
  }

  // ---- combine the waves' partial results: common reference = the largest one (wave 0 always has a tile) ----------
  s_ref[wv][l] = mrun;
  __syncthreads();
  float mall = s_ref[0][l];
#pragma unroll
  for (int k = 1; k < NS; ++k) mall = fmaxf(mall, s_ref[k][l]);
  const float sc = __builtin_amdgcn_exp2f(mrun - mall);       // 0 for a wave without tiles
  s_den[wv][l] = den * sc;
#pragma unroll
  for (int i = 0; i < DV / 32; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) s_acc[((size_t)wv * NR + 16 * i + v) * 64 + l] = acc[i][v] * sc;
  __syncthreads();
  float dsum = 0.0f;
#pragma unroll
  for (int k = 0; k < NS; ++k) dsum += s_den[k][l];
  const float dn = pair_sum(dsum);
  const bool ok = dn > 0.0f;
  const float inv = ok ? 1.0f / dn : 0.0f;
  // wave wv finishes accumulator registers [R wv, R (wv + 1)): register 16 i + v <-> column 32 i + 8 (v / 4) + 4 g + v % 4
  constexpr int R = NR / NS;
  if (q0 + c32 < m) {
    float *orow = out + ((size_t)bh * m + q0 + c32) * DV;
#pragma unroll
    for (int q4 = 0; q4 < R / 4; ++q4) {
      const int reg = R * wv + 4 * q4, i = reg / 16, v = reg % 16, col = 32 * i + 8 * (v / 4) + 4 * g;
      const float4 lo = *reinterpret_cast<const float4 *>(vmin + (size_t)pr * DV + col);
      const float4 hi = *reinterpret_cast<const float4 *>(vmax + (size_t)pr * DV + col);
      float o[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float a = 0.0f;
#pragma unroll
        for (int k = 0; k < NS; ++k) a += s_acc[((size_t)k * NR + reg + e) * 64 + l];
        o[e] = ok ? a * inv : 0.0f;
      }
      float4 res;
      res.x = fminf(fmaxf(o[0], lo.x), hi.x);
      res.y = fminf(fmaxf(o[1], lo.y), hi.y);
      res.z = fminf(fmaxf(o[2], lo.z), hi.z);
      res.w = fminf(fmaxf(o[3], lo.w), hi.w);
      *reinterpret_cast<float4 *>(orow + col) = res;
    }
  }
}

template <int D, int DV, int NS>
int launch_f32_split(const Shape &s, const void *Q, const wildcat_coreset *cs, void *out, float scale) {
  const size_t lds = (size_t)NS * (DV / 2) * 64 * sizeof(float);
  const void *fn = (const void *)k_wtd_attn_f32_split<D, DV, NS>;
  if (lds + 2 * NS * 64 * sizeof(float) > 64 * 1024 &&
      hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
    return WILDCAT_EHIP;
  hipLaunchKernelGGL((k_wtd_attn_f32_split<D, DV, NS>), dim3((unsigned)((s.m + 31) / 32), (unsigned)(s.batch * s.q_heads)),
                     dim3(NS * 64), lds, s.stream, (const float *)Q, (const float *)cs->k_s, cs->v_s, cs->w, cs->v_min,
                     cs->v_max, cs->r_eff, (float *)out, s.m, s.r, s.q_heads, s.group, scale);
  return hipGetLastError() == hipSuccess ? WILDCAT_OK : WILDCAT_EHIP;
}

template <int D, int DV>
int launch_mfma_f32(const Shape &s, const void *Q, const wildcat_coreset *cs, void *out) {
  const float scale = (float)(s.beta * (double)kLog2e);
  const int64_t heads = (int64_t)s.batch * s.q_heads;
  // Few queries in all and a coreset of several tiles: the waves of a workgroup share out the tiles (see above).
  if constexpr (DV <= 128) {
    const int64_t blocks = (s.m + 31) / 32 * heads;           // blocks of 32 queries
    const int tiles = (s.r + kFT - 1) / kFT;
    const int64_t cus = compute_units();
    if (blocks < 8 * cus && tiles >= 2) {
      // As many waves per block as there are tiles to share out, but not so many that the workgroups no longer run
      // all at once (two waves per SIMD, i.e. eight per compute unit, and the merge buffer in LDS): a second round of
      // workgroups costs more than longer chains of tiles per wave.
      auto one_round = [&](int ns) {
        const int64_t lds = (int64_t)ns * (DV / 2) * 256 + ns * 512 + 1024;
        const int64_t by_regs = 8 / ns, by_lds = 160 * 1024 / lds;
        return blocks <= (by_regs < by_lds ? by_regs : by_lds) * cus;
      };
      if (tiles >= 6 && one_round(8)) return launch_f32_split<D, DV, 8>(s, Q, cs, out, scale);
      if (tiles >= 3 && one_round(4)) return launch_f32_split<D, DV, 4>(s, Q, cs, out, scale);
      return launch_f32_split<D, DV, 2>(s, Q, cs, out, scale);
    }
  }
  // 128 queries per workgroup where that still gives every compute unit two workgroups, else 64
  const bool wide = DV == 256 || (s.m + 127) / 128 * heads >= 2 * (int64_t)compute_units();
  if (wide) {
    hipLaunchKernelGGL((k_wtd_attn_mfma_f32<D, DV, 4>), dim3((unsigned)((s.m + 127) / 128), (unsigned)heads), dim3(256),
                       0, s.stream, (const float *)Q, (const float *)cs->k_s, cs->v_s, cs->w, cs->v_min, cs->v_max,
                       cs->r_eff, (float *)out, s.m, s.r, s.q_heads, s.group, scale);
  } else {
    hipLaunchKernelGGL((k_wtd_attn_mfma_f32<D, DV, 2>), dim3((unsigned)((s.m + 63) / 64), (unsigned)heads), dim3(128),
                       0, s.stream, (const float *)Q, (const float *)cs->k_s, cs->v_s, cs->w, cs->v_min, cs->v_max,
                       cs->r_eff, (float *)out, s.m, s.r, s.q_heads, s.group, scale);
  }
  return hipGetLastError() == hipSuccess ? WILDCAT_OK : WILDCAT_EHIP;
}

// ---- packed values: v_t[pr][c][j] = fp16(v_s[pr][j][c] / v_scale[pr]) for j < r, zero for r <= j < r64 -----------
// v_scale[pr] = 2^(e - 14) with e the exponent of max |v_s[pr]|: the largest packed magnitude lies in [2^14, 2^15),
// inside fp16's range with the full significand for everything within 2^-28 of it.  Two small launches: the scale
// (one workgroup per problem, so no atomics and nothing to clear), then the packing.
__device__ __forceinline__ float value_scale(uint32_t max_bits) {
  const int e = (int)(max_bits >> 23);                      // biased exponent of the maximum
  if (e == 0 || e == 255) return 1.0f;                      // zero / subnormal / infinite maximum: no scaling
  const int se = min(max(e - 14, 1), 254);
  return __uint_as_float((uint32_t)se << 23);
}

constexpr int kScaleThreads = 1024;

__global__ __launch_bounds__(kScaleThreads) void k_value_scale(const float *__restrict__ v_s, int count,
                                                               float *__restrict__ v_scale) {
  __shared__ uint32_t sm[kScaleThreads / kWave];
  const int pr = blockIdx.x, t = threadIdx.x;
  const float *src = v_s + (size_t)pr * count;
  uint32_t b = 0u;
  for (int g0 = t; g0 < count; g0 += 8 * kScaleThreads) {   // eight loads in flight per thread
    uint32_t x[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int gid = g0 + q * kScaleThreads;
      x[q] = gid < count ? __float_as_uint(src[gid]) & 0x7fffffffu : 0u;
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      if (x[q] > 0x7f800000u) x[q] = 0u;                    // NaN: ignored
      b = b > x[q] ? b : x[q];
    }
  }
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) {
    const uint32_t o = __shfl_xor(b, off, kWave);
    b = b > o ? b : o;
  }
  if (t % kWave == 0) sm[t / kWave] = b;
  __syncthreads();
  if (t == 0) {
    for (int k = 1; k < kScaleThreads / kWave; ++k) b = b > sm[k] ? b : sm[k];
    v_scale[pr] = value_scale(b);
  }
}

__global__ __launch_bounds__(kThreads) void k_pack_values(const float *__restrict__ v_s,
                                                          const float *__restrict__ v_scale, int r, int r64, int dv,
                                                          uint16_t *__restrict__ v_t) {
  const int pr = blockIdx.y;
  const int gid = blockIdx.x * kThreads + threadIdx.x;
  if (gid >= r64 * dv) return;
  const int c = gid / r64, j = gid % r64;
  const float inv = 1.0f / v_scale[pr];                     // exact: a power of two
  const _Float16 h = (_Float16)(j < r ? v_s[((size_t)pr * r + j) * dv + c] * inv : 0.0f);   // round to nearest even
  v_t[((size_t)pr * dv + c) * r64 + j] = *reinterpret_cast<const uint16_t *>(&h);
}

// Both steps in one launch for small coresets (the binned and image-model shapes, where every launch of a few
// microseconds counts): one workgroup per problem finds the maximum, then packs.  Same values as the two kernels above.
__global__ __launch_bounds__(kScaleThreads) void k_scale_and_pack_values(const float *__restrict__ v_s, int r, int r64,
                                                                         int dv, float *__restrict__ v_scale,
                                                                         uint16_t *__restrict__ v_t) {
  __shared__ uint32_t sm[kScaleThreads / kWave];
  const int pr = blockIdx.x, t = threadIdx.x, count = r * dv;
  const float *src = v_s + (size_t)pr * count;
  uint32_t b = 0u;
  for (int gid = t; gid < count; gid += kScaleThreads) {
    uint32_t x = __float_as_uint(src[gid]) & 0x7fffffffu;
    if (x > 0x7f800000u) x = 0u;                            // NaN: ignored
    b = b > x ? b : x;
  }
#pragma unroll
  for (int off = kWave / 2; off > 0; off >>= 1) {
    const uint32_t o = __shfl_xor(b, off, kWave);
    b = b > o ? b : o;
  }
  if (t % kWave == 0) sm[t / kWave] = b;
  __syncthreads();
  b = sm[0];
  for (int k = 1; k < kScaleThreads / kWave; ++k) b = b > sm[k] ? b : sm[k];
  const float scale = value_scale(b);
  if (t == 0) v_scale[pr] = scale;
  const float inv = 1.0f / scale;                           // exact: a power of two
  for (int gid = t; gid < r64 * dv; gid += kScaleThreads) {
    const int c = gid / r64, j = gid % r64;
    const _Float16 h = (_Float16)(j < r ? src[(size_t)j * dv + c] * inv : 0.0f);   // round to nearest even
    v_t[((size_t)pr * dv + c) * r64 + j] = *reinterpret_cast<const uint16_t *>(&h);
  }
}

template <int D, int DV>
int launch_mfma2(const Shape &s, const void *Q, const wildcat_coreset *cs, void *out) {
  constexpr int NW = attn_waves<D, DV>();
  const int r64 = (s.r + 63) / 64 * 64;
  const int64_t qtiles = (s.m + NW * 32 - 1) / (NW * 32);
  const int64_t total = qtiles * s.batch * s.q_heads;
  if (total > INT32_MAX) return WILDCAT_EUNSUPPORTED;
  // Persistent grid: as many workgroups as fit on the device at once.
  int occ = 0;
  const int per_cu = (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, (const void *)k_wtd_attn_mfma2<D, DV, NW>,
                                                                   NW * 64, 0) == hipSuccess && occ >= 1) ? occ : 8 / NW;
  const int64_t resident = (int64_t)compute_units() * per_cu;
  const unsigned grid = (unsigned)(total < resident ? total : resident);
  hipLaunchKernelGGL((k_wtd_attn_mfma2<D, DV, NW>), dim3(grid), dim3(NW * 64), 0, s.stream, (const bf16_t *)Q,
                     (const bf16_t *)cs->k_s, (const uint16_t *)cs->v_t, cs->v_scale, cs->w, cs->v_min, cs->v_max, cs->r_eff,
                     (bf16_t *)out, s.m, s.r, r64, s.q_heads, s.group, (int)qtiles, (int)total,
                     (float)(s.beta * (double)kLog2e));
  return hipGetLastError() == hipSuccess ? WILDCAT_OK : WILDCAT_EHIP;
}

template <typename T>
int launch_simple(const Shape &s, const void *Q, const wildcat_coreset *cs, void *out) {
  const dim3 grid((unsigned)((s.m + kSQ - 1) / kSQ), s.batch * s.q_heads);
  const size_t lds = sizeof(float) * ((size_t)(kSQ + kSK) * (s.d + 1) + (size_t)kSK * s.dv + kSK + kSQ * kSK);
  hipLaunchKernelGGL((k_wtd_attn_simple<T>), grid, dim3(kThreads), lds, s.stream, (const T *)Q, (const T *)cs->k_s,
                     cs->v_s, cs->w, cs->v_min, cs->v_max, cs->r_eff, (T *)out, s.m, s.d, s.dv, s.r, s.q_heads, s.group,
                     (float)s.beta);
  return hipGetLastError() == hipSuccess ? WILDCAT_OK : WILDCAT_EHIP;
}

}  // namespace

int enqueue_pack_values(int P, int r, int dv, const float *v_s, void *v_t, float *v_scale, hipStream_t stream) {
  const int r64 = (r + 63) / 64 * 64;
  if ((int64_t)r64 * dv <= 16 * kScaleThreads) {             // at most sixteen elements per thread and phase
    hipLaunchKernelGGL(k_scale_and_pack_values, dim3(P), dim3(kScaleThreads), 0, stream, v_s, r, r64, dv, v_scale,
                       (uint16_t *)v_t);
    return hipGetLastError() == hipSuccess ? WILDCAT_OK : WILDCAT_EHIP;
  }
  hipLaunchKernelGGL(k_value_scale, dim3(P), dim3(kScaleThreads), 0, stream, v_s, r * dv, v_scale);
  hipLaunchKernelGGL(k_pack_values, dim3((r64 * dv + kThreads - 1) / kThreads, P), dim3(kThreads), 0, stream, v_s,
                     (const float *)v_scale, r, r64, dv, (uint16_t *)v_t);
  return hipGetLastError() == hipSuccess ? WILDCAT_OK : WILDCAT_EHIP;
}

}  // namespace wildcat

using namespace wildcat;

// ---- scratch that belongs to the library (wildcat_query_radius_static) ------------------------------------------
// Per-workgroup maxima of squared norms for callers that cannot hand over a workspace.  Every device the library
// runs on holds its own copy of this array, at its own address, until the process ends.  In host code the name
// below is only a handle for hipGetSymbolAddress; the address the kernels get is looked up once per device.
constexpr int kStaticHeads = 4096;                           // largest batch * q_heads the static entry point takes
constexpr int kStaticPartials = 4096 + kStaticHeads;         // doubles: 64 KB
static __device__ __align__(256) double scratch[kStaticPartials];

constexpr int kMaxDevices = 64;
static std::atomic<double *> scratch_ptr[kMaxDevices];       // per device; racing first calls store the same value

static int static_scratch(double **ptr) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return WILDCAT_EHIP;
  if (dev < 0 || dev >= kMaxDevices) return WILDCAT_EUNSUPPORTED;
  double *p = scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    void *sym = nullptr;
    if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return WILDCAT_EHIP;
    p = static_cast<double *>(sym);
    scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return WILDCAT_OK;
}

// Shared body of the two query-radius entry points.  `partial` (may be null): device memory for one double per
// workgroup, `partial_doubles` of them; `own_scratch`: the buffer is the library's (then a shape that does not fit
// is an error instead of a reason to fall back to atomics).
static int query_radius_impl(const void *Q, int64_t m, int32_t d, const wildcat_opts *opts, double *r_q_out,
                             double *partial_buf, size_t partial_doubles, bool own_scratch) {
  if (!Q || !r_q_out || m < 1) return WILDCAT_EINVAL;
  Shape s;
  int rc = resolve_shape(m, m, d, 1, opts, &s);
  if (rc != WILDCAT_OK) return rc;
  const int es = s.dtype == WILDCAT_BF16 ? 2 : 4;
  const int pieces = (d * es) % 16 == 0 ? d * es / 16 : 0;
  const bool vec = pieces >= 1 && pieces <= kWave && (pieces & (pieces - 1)) == 0;
  const int rows_per_pass = vec ? kThreads / pieces : kThreads;
  int64_t blocks = (m + rows_per_pass - 1) / rows_per_pass;
  const int64_t heads = (int64_t)s.batch * s.q_heads;
  const int64_t cap = (4096 + heads - 1) / heads;
  if (blocks > cap) blocks = cap;
  // Optional scratch (see wildcat_query_radius in wildcat.h): one double per workgroup.
  const size_t want = (size_t)heads * blocks;
  if (own_scratch && (heads > kStaticHeads || want > partial_doubles)) return WILDCAT_ETOOLARGE;
  double *partial = (vec && partial_buf && partial_doubles >= want) ? partial_buf : nullptr;
  if (!partial) {
    hipLaunchKernelGGL(k_zero_u64, dim3((s.P + 255) / 256), dim3(256), 0, s.stream, (unsigned long long *)r_q_out, s.P);
    if (hipGetLastError() != hipSuccess) return WILDCAT_EHIP;
  }
  if (vec) {
    const dim3 grid((unsigned)blocks, s.batch * s.q_heads);
    if (s.dtype == WILDCAT_BF16)
      hipLaunchKernelGGL((k_qnorm_max_vec<bf16_t>), grid, dim3(kThreads), 0, s.stream, (const bf16_t *)Q, m, d, pieces,
                         s.q_heads, s.group, (unsigned long long *)r_q_out, partial);
    else
      hipLaunchKernelGGL((k_qnorm_max_vec<float>), grid, dim3(kThreads), 0, s.stream, (const float *)Q, m, d, pieces,
                         s.q_heads, s.group, (unsigned long long *)r_q_out, partial);
    if (partial) {
      if (hipGetLastError() != hipSuccess) return WILDCAT_EHIP;
      hipLaunchKernelGGL(k_radius_final, dim3(s.P), dim3(kThreads), 0, s.stream, partial, (int)(s.group * blocks),
                         r_q_out);
    }
  } else {
    const dim3 grid((unsigned)((m + kThreads - 1) / kThreads), s.batch * s.q_heads);
    if (s.dtype == WILDCAT_BF16)
      hipLaunchKernelGGL((k_qnorm_max<bf16_t>), grid, dim3(kThreads), 0, s.stream, (const bf16_t *)Q, m, d, s.q_heads,
                         s.group, (unsigned long long *)r_q_out);
    else
      hipLaunchKernelGGL((k_qnorm_max<float>), grid, dim3(kThreads), 0, s.stream, (const float *)Q, m, d, s.q_heads,
                         s.group, (unsigned long long *)r_q_out);
  }
  return hipGetLastError() == hipSuccess ? WILDCAT_OK : WILDCAT_EHIP;
}

extern "C" int wildcat_query_radius(const void *Q, int64_t m, int32_t d, const wildcat_opts *opts, double *r_q_out) {
  double *buf = nullptr;
  size_t doubles = 0;
  if (opts && opts->workspace && !((uintptr_t)opts->workspace & 255)) {
    buf = (double *)opts->workspace;
    doubles = opts->workspace_bytes / sizeof(double);
  }
  return query_radius_impl(Q, m, d, opts, r_q_out, buf, doubles, false);
}

extern "C" int wildcat_query_radius_static(const void *Q, int64_t m, int32_t d, const wildcat_opts *opts,
                                           double *r_q_out) {
  double *buf = nullptr;
  const int rc = static_scratch(&buf);
  if (rc != WILDCAT_OK) return rc;
  return query_radius_impl(Q, m, d, opts, r_q_out, buf, (size_t)kStaticPartials, true);
}

extern "C" int wildcat_wtd_attn(const void *Q, const wildcat_coreset *cs, void *out, int64_t m, int32_t d, int32_t r,
                                const wildcat_opts *opts) {
  if (!Q || !cs || !out || m < 1 || r < 1) return WILDCAT_EINVAL;
  if (!cs->k_s || !cs->v_s || !cs->w || !cs->v_min || !cs->v_max) return WILDCAT_EINVAL;
  Shape s;
  int rc = resolve_shape(r, m, d, r, opts, &s);
  if (rc != WILDCAT_OK) return rc;
  // With bins, an exhausted bin leaves empty slots in the middle of the coreset (zero key, value and weight: they
  // add nothing), so every slot is read and cs->r_eff, which is then per bin, is not consulted.
  wildcat_coreset all_slots;
  if (s.bins > 1) {
    all_slots = *cs;
    all_slots.r_eff = nullptr;
    cs = &all_slots;
  }
  if (s.dtype == WILDCAT_BF16) {
    // the MFMA kernel addresses a problem's packed values with 32-bit byte offsets
    const bool fits = (int64_t)((s.r + 63) / 64 * 64) * s.dv * 2 <= (int64_t)UINT32_MAX;
    if (cs->v_t && cs->v_scale && fits) {
      // decode shape: so few packed rows per kv head that splitting the keys over the waves of a workgroup beats
      // giving every head a workgroup of its own
      // (as long as that leaves compute units idle: its operands come straight from memory, which costs more per
      // tile than the staged tiles of the kernel above once there is enough work to fill the device)
      const int64_t packed_rows = (int64_t)s.group * s.m;
      if (packed_rows <= kDecodeRows && (packed_rows + 31) / 32 * s.P <= compute_units()) {
        if (s.d == 64 && s.dv == 64) return launch_decode<64, 64>(s, Q, cs, out);
        if (s.d == 128 && s.dv == 128) return launch_decode<128, 128>(s, Q, cs, out);
      }
      if (s.d == 64 && s.dv == 64) return launch_mfma2<64, 64>(s, Q, cs, out);
      if (s.d == 128 && s.dv == 128) return launch_mfma2<128, 128>(s, Q, cs, out);
      if (s.d == 64 && s.dv == 128) return launch_mfma2<64, 128>(s, Q, cs, out);
      if (s.d == 128 && s.dv == 64) return launch_mfma2<128, 64>(s, Q, cs, out);
      if (s.d == 64 && s.dv == 256) return launch_mfma2<64, 256>(s, Q, cs, out);
    }
    return launch_simple<bf16_t>(s, Q, cs, out);
  }
  if (s.batch * s.q_heads <= 65535) {
    if (s.d == 64 && s.dv == 64) return launch_mfma_f32<64, 64>(s, Q, cs, out);
    if (s.d == 64 && s.dv == 256) return launch_mfma_f32<64, 256>(s, Q, cs, out);
    if (s.d == 128 && s.dv == 128) return launch_mfma_f32<128, 128>(s, Q, cs, out);
  }
  return launch_simple<float>(s, Q, cs, out);
}

extern "C" int wildcat_pack_values(const wildcat_coreset *cs, int32_t r, int32_t dv, const wildcat_opts *opts) {
  if (!cs || !cs->v_s || !cs->v_t || !cs->v_scale || r < 1 || dv < 1) return WILDCAT_EINVAL;
  Shape s;
  int rc = resolve_shape(r, 0, dv, r, opts, &s);
  if (rc != WILDCAT_OK) return rc;
  if (s.dtype != WILDCAT_BF16) return WILDCAT_EINVAL;
  return enqueue_pack_values(s.P, r, dv, cs->v_s, cs->v_t, cs->v_scale, s.stream);
}
