// CompressKV (Alg. 2) with the RPNys selection loop (Alg. 1) for gfx950.
//
// Bins (Sec. 2.5) are handled as a batch: B contiguous bins of n/B keys are a reshape of K and V, so every kernel
// below simply sees P * B problems of n/B keys and r/B pivots ("problem" = one bin of one (batch, kv head) pair).
// Only three things know about the grouping: the key mean and the value range are taken over all bins of a head
// (k_col_final), the temperature reads R_Q of the bin's head (k_init_p), and pivot indices are made global at the end.
//
// The selection loop is bound by HBM bandwidth: step i must touch, for every key l, the i numbers
// already computed for that key.  Everything here is laid out so that this stream is contiguous and
// read with full-width loads:
//
//   * Keys are re-packed once as Kp[problem][d/4][n][4], so a thread that owns one or two adjacent keys
//     reads 8..32 contiguous bytes per 4-wide chunk of the feature dimension and a wavefront reads a
//     contiguous run.
//   * Instead of the kernel rows R and the explicit inverse M of Alg. 1, the loop keeps the partial
//     Cholesky rows F_i(l) = h_res^{i}(k_s, k_l) / sqrt(h_res^{i}(k_s, k_s)); delta of Alg. 1 equals
//     -F_i (proof of Thm. 1), so p <- p - delta^2 is p <- p - F_i^2, the lower-triangular L with
//     L[j][i] = F_i(s_j) satisfies h(K_S,K_S) = L L^T (so M = L^-T L^-1), and W = M R = L^-T F.
//     Same pivots in exact arithmetic, same bytes per step, better conditioned than updating M.
//   * F is stored slab-blocked, F[problem][slab][r][slab_keys]: the history of a workgroup's keys is one
//     contiguous region.
//   * All pivot-critical arithmetic (inner products, exp, history, p, prefix sums, the comparison
//     against u * sum p) is fp64, so that the drawn index equals the one a float64 reference draws
//     from the same uniform.  Sums use a fixed order: results are bit-reproducible run to run.
//
//     (Fast mode, wildcat_history in wildcat.h: the history rows alone are stored in fp32.)
//
// Every workgroup redoes the (cheap) pivot search from the per-slab sums the previous step left.  The loop runs as
// one persistent launch whose workgroups synchronise through those sums when they all fit on the device, and as
// one launch per step otherwise (see rpnys_step and its two drivers).
#include <climits>
#include <cmath>

#include "common.h"

namespace wildcat {
namespace {

// --------------------------------------------------------------------------------------------
// Column statistics of K (sums, for the mean of Alg. 2) and V (min / max, Alg. 4), pass 1.
// grid (nb0, P); thread (rr, cc) walks rows rr, rr+rif, ... of its row block, column cc.
// --------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void k_col_stats(const T *__restrict__ K, const T *__restrict__ V,
                                                        int64_t n, int d, int dv, int dpad, int nb0, int lpr,
                                                        double *__restrict__ mpart, float *__restrict__ vminpart,
                                                        float *__restrict__ vmaxpart) {
  __shared__ double sd[kThreads];
  __shared__ float smn[kThreads], smx[kThreads];
  const int t = threadIdx.x, blk = blockIdx.x, pr = blockIdx.y;
  const int rif = kThreads / lpr, rr = t / lpr, cc = t % lpr;
  const int64_t rpb = (n + nb0 - 1) / nb0;
  const int64_t row0 = blk * rpb, row1 = (row0 + rpb < n) ? row0 + rpb : n;
  const T *Kp = K + (size_t)pr * n * d;
  const T *Vp = V + (size_t)pr * n * dv;
  double acc = 0.0;
  float mn = INFINITY, mx = -INFINITY;
  for (int64_t row = row0 + rr; row < row1; row += rif) {
    if (cc < d) acc += (double)to_float(Kp[row * d + cc]);
    if (cc < dv) {
      float v = to_float(Vp[row * dv + cc]);
      mn = fminf(mn, v);
      mx = fmaxf(mx, v);
    }
  }
  sd[t] = acc; smn[t] = mn; smx[t] = mx;
  __syncthreads();
  if (rr == 0) {
    for (int q = 1; q < rif; ++q) {
      acc += sd[q * lpr + cc];
      mn = fminf(mn, smn[q * lpr + cc]);
      mx = fmaxf(mx, smx[q * lpr + cc]);
    }
    if (cc < dpad) mpart[((size_t)pr * nb0 + blk) * dpad + cc] = cc < d ? acc : 0.0;
    if (cc < dv) {
      vminpart[((size_t)pr * nb0 + blk) * dv + cc] = mn;
      vmaxpart[((size_t)pr * nb0 + blk) * dv + cc] = mx;
    }
  }
}

// pass 2.  The mean of Alg. 2 and the value range of Alg. 4 belong to the whole head: they are combined over the
// `bins` consecutive problems of the head in a fixed order -- logical thread (rr, cc) of kFinalThreads / lpr x lpr
// takes partials rr, rr + rif, ... of column cc, eight loads in flight at a time, then the rif partial results are
// added in turn -- and kbar is written once per bin so that later kernels index it by problem.  n = keys per bin.
// The lpr columns are dealt out to gridDim.y workgroups of kFinalThreads / gridDim.y threads (a slice of lpr /
// gridDim.y columns each, every thread doing what its logical thread does: the same bits whatever the slicing), so
// that several compute units share the reading.  grid (heads, slices).  Clears the R_K^2 accumulators of the head's bins.
constexpr int kFinalThreads = 1024;

__global__ __launch_bounds__(kFinalThreads) void k_col_final(const double *__restrict__ mpart,
                                                             const float *__restrict__ vminpart,
                                                             const float *__restrict__ vmaxpart, int64_t n, int dv,
                                                             int dpad, int nb0, int bins, int lpr,
                                                             double *__restrict__ kbar, float *__restrict__ vmin,
                                                             float *__restrict__ vmax,
                                                             unsigned long long *__restrict__ scal) {
  __shared__ double sd[kFinalThreads];
  __shared__ float smn[kFinalThreads], smx[kFinalThreads];
  const int t = threadIdx.x, head = blockIdx.x, nthr = blockDim.x;
  const int lprs = lpr / gridDim.y, c0 = blockIdx.y * lprs;   // this workgroup's columns: c0 .. c0 + lprs - 1
  const int rif = kFinalThreads / lpr, rr = t / lprs, cl = t % lprs, cc = c0 + cl;
  const size_t part0 = (size_t)head * bins * nb0;
  const int nparts = bins * nb0;
  double acc = 0.0;
  float mn = INFINITY, mx = -INFINITY;
  for (int b0 = rr; b0 < nparts; b0 += 8 * rif) {
    double x[8];
    float lo[8], hi[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int b = b0 + q * rif;
      const bool ok = b < nparts;
      x[q] = (ok && cc < dpad) ? mpart[(part0 + b) * dpad + cc] : 0.0;
      lo[q] = (ok && cc < dv) ? vminpart[(part0 + b) * dv + cc] : INFINITY;
      hi[q] = (ok && cc < dv) ? vmaxpart[(part0 + b) * dv + cc] : -INFINITY;
    }
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      acc += x[q];
      mn = fminf(mn, lo[q]);
      mx = fmaxf(mx, hi[q]);
    }
  }
  sd[t] = acc; smn[t] = mn; smx[t] = mx;
  __syncthreads();
  if (rr == 0) {
    for (int q = 1; q < rif; ++q) {
      acc += sd[q * lprs + cl];
      mn = fminf(mn, smn[q * lprs + cl]);
      mx = fmaxf(mx, smx[q * lprs + cl]);
    }
    if (cc < dv) {
      vmin[(size_t)head * dv + cc] = mn;
      vmax[(size_t)head * dv + cc] = mx;
    }
  }
  __syncthreads();                                           // (sd is read above by the threads of rr == 0 only)
  if (rr == 0) sd[cl] = acc / ((double)n * (double)bins);
  __syncthreads();
  for (int e = t; e < bins * lprs; e += nthr) {              // one copy of the mean per bin, written by everybody
    const int b = e / lprs, c = c0 + e % lprs;
    if (c < dpad) kbar[((size_t)head * bins + b) * dpad + c] = sd[e % lprs];
  }
  if (blockIdx.y == 0)
    for (int b = t; b < bins; b += nthr) scal[((size_t)head * bins + b) * 8] = 0ull;
}

// --------------------------------------------------------------------------------------------
// Re-pack keys: Kp[pr][c][l][e] = K[pr][l][4c+e] (zero beyond n or d).  grid (ceil(npad*nc/256), P).
// --------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(kThreads) void k_pack(const T *__restrict__ K, int64_t n, int64_t npad, int d,
                                                   int dpad, T *__restrict__ Kp) {
  const int pr = blockIdx.y, nc = dpad / kChunk;
  const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (gid >= npad * nc) return;
  const int64_t l = gid % npad;
  const int c = (int)(gid / npad);
  T out[kChunk];
#pragma unroll
  for (int e = 0; e < kChunk; ++e) {
    const int j = c * kChunk + e;
    T z;
    from_float(0.0f, &z);
    out[e] = (l < n && j < d) ? K[((size_t)pr * n + l) * d + j] : z;
  }
  T *dst = Kp + (((size_t)pr * nc + c) * npad + l) * kChunk;
#pragma unroll
  for (int e = 0; e < kChunk; ++e) dst[e] = out[e];
}

// --------------------------------------------------------------------------------------------
// Fused first pass for the common widths (rows of K and V that are a power-of-two number of 16-byte pieces):
// one read of K produces both the packed copy Kp and the column sums, one read of V the column minima and maxima.
// grid (nb, P); the workgroup owns keys [blk * kpw, (blk + 1) * kpw), kpw a multiple of the tile height.
//   * K rows are contiguous in memory, so a tile of TK rows is read as one linear run of 16-byte pieces (lane i of
//     a wavefront takes piece i), parked in LDS with an 8-byte row pad, and written back out chunk by chunk: for a
//     fixed chunk c the TK keys of the tile are contiguous in Kp, so stores are full lines too.
//   * A thread always holds the same piece column (256 is a multiple of the pieces per row), so the column sums,
//     minima and maxima accumulate in registers and are combined once at the end, in a fixed order.
// Same partial-result layout as k_col_stats (pass 2 is k_col_final).
// --------------------------------------------------------------------------------------------
template <typename T> struct Piece;                    // 16 bytes of a row as floats
template <> struct Piece<float> {
  static constexpr int N = 4;
  __device__ static void unpack(uint4 v, float (&x)[4]) {
    x[0] = __uint_as_float(v.x); x[1] = __uint_as_float(v.y); x[2] = __uint_as_float(v.z); x[3] = __uint_as_float(v.w);
  }
};
template <> struct Piece<bf16_t> {
  static constexpr int N = 8;
  __device__ static void unpack(uint4 v, float (&x)[8]) {
    x[0] = __uint_as_float(v.x << 16); x[1] = __uint_as_float(v.x & 0xffff0000u);
    x[2] = __uint_as_float(v.y << 16); x[3] = __uint_as_float(v.y & 0xffff0000u);
    x[4] = __uint_as_float(v.z << 16); x[5] = __uint_as_float(v.z & 0xffff0000u);
    x[6] = __uint_as_float(v.w << 16); x[7] = __uint_as_float(v.w & 0xffff0000u);
  }
};

template <typename T>
__global__ __launch_bounds__(kThreads) void k_pack_stats(const T *__restrict__ K, const T *__restrict__ V, int64_t n,
                                                         int64_t npad, int d, int dv, int kpw, int tk, int nb,
                                                         T *__restrict__ Kp, double *__restrict__ mpart,
                                                         float *__restrict__ vminpart, float *__restrict__ vmaxpart) {
  constexpr int EPP = Piece<T>::N;                       // elements per 16-byte piece
  extern __shared__ __attribute__((aligned(16))) char tile[];   // tk rows of (d * sizeof(T) + 8) bytes
  __shared__ double sks[kThreads / kWave][kMaxWidth];           // per wavefront and column
  __shared__ float smn[kThreads / kWave][kMaxWidth], smx[kThreads / kWave][kMaxWidth];
  const int t = threadIdx.x, blk = blockIdx.x, pr = blockIdx.y;
  const int ppr = d / EPP, ppv = dv / EPP;               // pieces per K row / V row (powers of two <= 64)
  const int rowb = d * (int)sizeof(T) + 8;
  const int nc = d / kChunk;
  const int64_t key0 = (int64_t)blk * kpw;
  const int64_t key1 = key0 + kpw < npad ? key0 + kpw : npad;
  const T *Kpr = K + (size_t)pr * n * d;

  // ---- K: pack and column sums ---------------------------------------------------------------------------
  const int jk = t % ppr, rk = t / ppr, rpp = kThreads / ppr;
  double ksum[EPP];
#pragma unroll
  for (int e = 0; e < EPP; ++e) ksum[e] = 0.0;
  // Tiles that lie wholly in the padding (rows >= n) are not written: with small bins the padding up to a full
  // slab is many times the data, and every reader of the packed copy skips rows >= n.
  // A thread's pieces of a tile (tk / rpp of them: at most kPackLoads) are fetched one tile ahead: the next tile's
  // loads are issued as soon as the current one has been copied to LDS, and fly while it is written out.
  constexpr int kPackLoads = 8;
  uint4 cur[kPackLoads];                                 // piece q of a thread: tile row rk + q rpp (if < tk)
  auto fetch = [&](int64_t tile0) {
#pragma unroll
    for (int q = 0; q < kPackLoads; ++q) {
      const int lr = rk + q * rpp;
      const int64_t row = tile0 + lr;
      cur[q] = make_uint4(0u, 0u, 0u, 0u);
      if (lr < tk && row < n) cur[q] = *reinterpret_cast<const uint4 *>(Kpr + (size_t)row * d + jk * EPP);
    }
  };
  if (key0 < key1 && key0 < n) fetch(key0);
  for (int64_t tile0 = key0; tile0 < key1 && tile0 < n; tile0 += tk) {
#pragma unroll
    for (int q = 0; q < kPackLoads; ++q) {
      const int lr = rk + q * rpp;
      if (lr < tk) {
        float x[EPP];
        Piece<T>::unpack(cur[q], x);
#pragma unroll
        for (int e = 0; e < EPP; ++e) ksum[e] += (double)x[e];
        uint2 *dst = reinterpret_cast<uint2 *>(tile + (size_t)lr * rowb + jk * 16);
        dst[0] = make_uint2(cur[q].x, cur[q].y);
        dst[1] = make_uint2(cur[q].z, cur[q].w);
      }
    }
    if (tile0 + tk < key1 && tile0 + tk < n) fetch(tile0 + tk);
    __syncthreads();
    for (int item = t; item < nc * tk; item += kThreads) {
      const int l = item % tk, c = item / tk;
      const char *src = tile + (size_t)l * rowb + c * (kChunk * (int)sizeof(T));
      T *dst = Kp + (((size_t)pr * nc + c) * npad + tile0 + l) * kChunk;
      if constexpr (sizeof(T) == 2) {
        *reinterpret_cast<uint2 *>(dst) = *reinterpret_cast<const uint2 *>(src);
      } else {
        const uint2 a = reinterpret_cast<const uint2 *>(src)[0], b = reinterpret_cast<const uint2 *>(src)[1];
        *reinterpret_cast<uint4 *>(dst) = make_uint4(a.x, a.y, b.x, b.y);
      }
    }
    __syncthreads();
  }

  // ---- V: column minima and maxima -------------------------------------------------------------------------
  const int jv = t % ppv, rv = t / ppv, rpv = kThreads / ppv;
  float mn[EPP], mx[EPP];
#pragma unroll
  for (int e = 0; e < EPP; ++e) { mn[e] = INFINITY; mx[e] = -INFINITY; }
  const T *Vpr = V + (size_t)pr * n * dv;
  const int64_t vend = key1 < n ? key1 : n;
#pragma unroll 4
  for (int64_t row = key0 + rv; row < vend; row += rpv) {
    const uint4 v = *reinterpret_cast<const uint4 *>(Vpr + (size_t)row * dv + jv * EPP);
    float x[EPP];
    Piece<T>::unpack(v, x);
#pragma unroll
    for (int e = 0; e < EPP; ++e) { mn[e] = fminf(mn[e], x[e]); mx[e] = fmaxf(mx[e], x[e]); }
  }

  // ---- combine the threads that share a piece column: the lanes of a wavefront by a butterfly over the lanes that
  // differ in the row group only (a fixed order), then the four wavefronts in turn ----------------------------------
  const int lane = t & (kWave - 1), wv = t / kWave;
  for (int off = ppr; off < kWave; off <<= 1)
#pragma unroll
    for (int e = 0; e < EPP; ++e) ksum[e] += __shfl_xor(ksum[e], off, kWave);
  for (int off = ppv; off < kWave; off <<= 1)
#pragma unroll
    for (int e = 0; e < EPP; ++e) {
      mn[e] = fminf(mn[e], __shfl_xor(mn[e], off, kWave));
      mx[e] = fmaxf(mx[e], __shfl_xor(mx[e], off, kWave));
    }
  if (lane < ppr)
#pragma unroll
    for (int e = 0; e < EPP; ++e) sks[wv][lane * EPP + e] = ksum[e];
  if (lane < ppv)
#pragma unroll
    for (int e = 0; e < EPP; ++e) { smn[wv][lane * EPP + e] = mn[e]; smx[wv][lane * EPP + e] = mx[e]; }
  __syncthreads();
  const size_t slot = (size_t)pr * nb + blk;
  if (t < d) {
    double acc = 0.0;
    for (int q = 0; q < kThreads / kWave; ++q) acc += sks[q][t];
    mpart[slot * d + t] = acc;
  }
  if (t < dv) {
    float lo = INFINITY, hi = -INFINITY;
    for (int q = 0; q < kThreads / kWave; ++q) {
      lo = fminf(lo, smn[q][t]);
      hi = fmaxf(hi, smx[q][t]);
    }
    vminpart[slot * dv + t] = lo;
    vmaxpart[slot * dv + t] = hi;
  }
}

// Loads the kChunk packed features of KPT adjacent keys as floats.
template <typename T, int KPT>
__device__ __forceinline__ void load_chunk(const T *__restrict__ src, float (&x)[KPT][kChunk]);

template <>
__device__ __forceinline__ void load_chunk<float, 1>(const float *__restrict__ src, float (&x)[1][kChunk]) {
  const float4 v = *reinterpret_cast<const float4 *>(src);
  x[0][0] = v.x; x[0][1] = v.y; x[0][2] = v.z; x[0][3] = v.w;
}
template <>
__device__ __forceinline__ void load_chunk<float, 2>(const float *__restrict__ src, float (&x)[2][kChunk]) {
  const float4 a = reinterpret_cast<const float4 *>(src)[0], b = reinterpret_cast<const float4 *>(src)[1];
  x[0][0] = a.x; x[0][1] = a.y; x[0][2] = a.z; x[0][3] = a.w;
  x[1][0] = b.x; x[1][1] = b.y; x[1][2] = b.z; x[1][3] = b.w;
}
__device__ __forceinline__ void unpack_bf16x4(uint2 v, float (&x)[kChunk]) {
  x[0] = __uint_as_float(v.x << 16); x[1] = __uint_as_float(v.x & 0xffff0000u);
  x[2] = __uint_as_float(v.y << 16); x[3] = __uint_as_float(v.y & 0xffff0000u);
}
template <>
__device__ __forceinline__ void load_chunk<bf16_t, 1>(const bf16_t *__restrict__ src, float (&x)[1][kChunk]) {
  unpack_bf16x4(*reinterpret_cast<const uint2 *>(src), x[0]);
}
template <>
__device__ __forceinline__ void load_chunk<bf16_t, 2>(const bf16_t *__restrict__ src, float (&x)[2][kChunk]) {
  const uint4 v = *reinterpret_cast<const uint4 *>(src);
  unpack_bf16x4(make_uint2(v.x, v.y), x[0]);
  unpack_bf16x4(make_uint2(v.z, v.w), x[1]);
}

// --------------------------------------------------------------------------------------------
// sq[l] = ||k_l - kbar||^2 (fp64) and R_K^2 = max_l sq[l] (Alg. 2, first line of the bin loop).
// grid (nblk, P).  The maximum of non-negative doubles is taken on their bit patterns, which order
// the same way, with an integer atomic: exact and order-independent.
// --------------------------------------------------------------------------------------------
template <typename T, int KPT>
__global__ __launch_bounds__(kThreads) void k_sqnorm(const T *__restrict__ Kp, const double *__restrict__ kbar,
                                                     int64_t n, int64_t npad, int dpad, double *__restrict__ sq,
                                                     unsigned long long *__restrict__ scal) {
  __shared__ double skb[kMaxWidth];
  __shared__ double sm[kThreads / kWave];
  const int t = threadIdx.x, b = blockIdx.x, pr = blockIdx.y, nc = dpad / kChunk;
  if (t < dpad) skb[t] = kbar[(size_t)pr * dpad + t];
  __syncthreads();
  const int64_t l0 = (int64_t)b * (kThreads * KPT) + t * KPT;
  double acc[KPT];
#pragma unroll
  for (int k = 0; k < KPT; ++k) acc[k] = 0.0;
  if (l0 < n) {                                              // padding rows of the packed copy are not even written
    for (int c = 0; c < nc; ++c) {
      float x[KPT][kChunk];
      load_chunk<T, KPT>(Kp + (((size_t)pr * nc + c) * npad + l0) * kChunk, x);
#pragma unroll
      for (int k = 0; k < KPT; ++k)
#pragma unroll
        for (int e = 0; e < kChunk; ++e) {
          const double df = (double)x[k][e] - skb[c * kChunk + e];
          acc[k] = fma(df, df, acc[k]);
        }
    }
  }
  double mx = 0.0;
#pragma unroll
  for (int k = 0; k < KPT; ++k) {
    if (l0 + k >= n) acc[k] = 0.0;
    sq[(size_t)pr * npad + l0 + k] = acc[k];
    mx = fmax(mx, acc[k]);
  }
  mx = block_reduce<double>(mx, sm, MaxOp());
  if (t == 0) {
    // The accumulator only grows, so a workgroup whose maximum is not above what is already there has nothing to
    // add (a stale read merely costs an atomic that changes nothing): most workgroups skip the contended atomic.
    const unsigned long long bits = (unsigned long long)__double_as_longlong(mx);
    if (bits > __hip_atomic_load(&scal[(size_t)pr * 8], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
      atomicMax(&scal[(size_t)pr * 8], bits);
  }
}

// --------------------------------------------------------------------------------------------
// Temperature, eq. (kernel-temperature):  b0 = log n / (beta R_Q R_K) + 2,
// rho = b0 / (2 W0(b0 / (2 rho0))), tau = sqrt(rho R_K / R_Q); the loop then uses beta / tau^2.
// W0 by Newton on w + log w = log z (z = b0 / (2 rho0) > 0.3 here).
// If R_K or R_Q is zero every kernel value is 1 whatever tau is; tau is then reported as +inf and
// the loop runs with exponent scale 0.
// --------------------------------------------------------------------------------------------
// One thread evaluates this while its workgroup waits, so the chain of double-precision logarithms is kept short:
// the start comes from a few single-precision rounds, and the iteration stops once a step is below 1e-9 relative --
// Newton converges quadratically here (error_next <= 1.9 error^2 for w >= 0.2), so the value after that step is
// exact to rounding.
__device__ __forceinline__ double lambert_w0(double z) {
  float wf = log1pf((float)z);
  const float lzf = logf((float)z);
  for (int it = 0; it < 4; ++it) wf -= (wf + logf(wf) - lzf) / (1.0f + 1.0f / wf);
  const double lz = log(z);
  double w = wf > 0.0f && wf < INFINITY ? (double)wf : log1p(z);
  for (int it = 0; it < 64; ++it) {
    const double wn = w - (w + log(w) - lz) / (1.0 + 1.0 / w);
    const bool done = fabs(wn - w) <= 1e-9 * fabs(wn);
    w = wn;
    if (done) break;
  }
  return w;
}

// rho_0 = sqrt(1 + exp(W0(2 / e^2) + 2)) = sqrt(1 + 2 / W0(2 / e^2))   (eq. (kernel-temperature)), W0(2 / e^2) =
// 0.21771510575709011...
constexpr double kRho0 = 0x1.988661e4d29bbp+1;               // 3.19160102532370412...

// Evaluated by one thread of every workgroup of k_init_p (same inputs, same arithmetic, same value everywhere).
__device__ __forceinline__ void temperature(double rk2, double rq, double n, double beta, double *tau, double *beta_tau, double *rk_out) {
  const double rk = sqrt(rk2);
  if (!(rk > 0.0) || !(rq > 0.0)) {
    *tau = INFINITY;
    *beta_tau = 0.0;
  } else {
    const double b0 = log(n) / (beta * rq * rk) + 2.0;
    const double rho = b0 / (2.0 * lambert_w0(b0 / (2.0 * kRho0)));
    *tau = sqrt(rho * rk / rq);
    *beta_tau = beta / (*tau * *tau);
  }
  *rk_out = rk;
}

// --------------------------------------------------------------------------------------------
// The temperature of the problem (bin) from its R_K^2 (scal[8 pr], left by k_sqnorm) and the R_Q of its head, then
// Alg. 1, first line: p_l = h_tau(k_l, k_l) = exp(beta_tau ||k_l - kbar||^2); also the per-key floor
// rank_tol * p_l, the per-slab sums, idx = -1, r_eff = r and (if asked) the uniforms of the seed.
// grid (nblk, P).  sq_floor holds sq on entry and the floor on exit.  Workgroup 0 of a problem records tau,
// beta / tau^2 and R_K in scal[8 pr + 1 .. 3] and tau in tau_out.  tau_n = the sequence length that enters b0.
// --------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned long long mix64(unsigned long long z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

template <int KPT>
__global__ __launch_bounds__(kThreads) void k_init_p(int64_t n, int64_t npad, int nblk, int r, double rank_tol,
                                                     int bins, double tau_n, double beta,
                                                     const double *__restrict__ r_q, double *__restrict__ scal,
                                                     double *__restrict__ tau_out, double *__restrict__ sq_floor,
                                                     double *__restrict__ p0, double *__restrict__ bsum0,
                                                     int32_t *__restrict__ idx, int32_t *__restrict__ r_eff,
                                                     double *__restrict__ u_gen, unsigned long long seed,
                                                     int *__restrict__ sync_error, long long *__restrict__ mail,
                                                     long long mail_per_problem) {
  __shared__ double sm[kThreads / kWave];
  __shared__ double s_beta_tau;
  const int t = threadIdx.x, b = blockIdx.x, pr = blockIdx.y;
  if (t == 0) {
    double tau, bt, rk;
    temperature(__longlong_as_double(((const long long *)scal)[(size_t)pr * 8]), r_q[pr / bins], tau_n, beta, &tau, &bt,
                &rk);
    s_beta_tau = bt;
    if (b == 0) {
      scal[(size_t)pr * 8 + 1] = tau;
      scal[(size_t)pr * 8 + 2] = bt;
      scal[(size_t)pr * 8 + 3] = rk;
      tau_out[pr] = tau;
    }
  }
  __syncthreads();
  const double beta_tau = s_beta_tau;
  const int64_t l0 = (int64_t)b * (kThreads * KPT) + t * KPT;
  double loc = 0.0;
#pragma unroll
  for (int k = 0; k < KPT; ++k) {
    const size_t at = (size_t)pr * npad + l0 + k;
    const double v = (l0 + k < n) ? exp(beta_tau * sq_floor[at]) : 0.0;
    p0[at] = v;
    sq_floor[at] = rank_tol * v;
    loc += v;
  }
  const double tot = block_sum(loc, sm);
  double *bs = bsum0 + (size_t)pr * r * nblk;               // [r][nblk]: row 0 = initial sums, the rest unpublished
  if (t == 0) bs[b] = tot;
  for (int i = 1 + t; i < r; i += kThreads) bs[(size_t)i * nblk + b] = -1.0;
  if (mail)                                                  // pivot records of the resident loop: nothing has arrived
    for (long long w = (long long)b * kThreads + t; w < mail_per_problem; w += (long long)nblk * kThreads)
      mail[(size_t)pr * mail_per_problem + w] = kMailEmpty;
  if (b == 0) {
    for (int i = t; i < r; i += kThreads) {
      idx[(size_t)pr * r + i] = -1;
      if (u_gen) {
        const unsigned long long ctr = (unsigned long long)pr * r + i + 1ull;
        u_gen[(size_t)pr * r + i] = (double)(mix64(seed + ctr * 0x9E3779B97F4A7C15ull) >> 11) * 0x1.0p-53;
      }
    }
    if (t == 0) {
      r_eff[pr] = r;
      if (pr == 0) *sync_error = 0;
    }
  }
}

// --------------------------------------------------------------------------------------------
// One RPNys step (body of the loop of Alg. 1) for step index i, as a device function shared by the two
// drivers below: `k_step` (one launch per step, grid (nblk, P)) and `k_rpnys_persistent` (one launch for the
// whole loop, workgroups of a problem synchronising through the per-slab sums).
// --------------------------------------------------------------------------------------------
struct StepArgs {
  const void *Kp;         // [P][dpad/4][npad][4] packed keys
  const double *kbar;     // [P][dpad]
  const double *scal;     // [P][8]: 1 = tau, 2 = beta_tau
  const double *floor;    // [P][npad]
  const double *u;        // [P][r]
  double *p;              // [2][P][npad]   residual diagonal, double-buffered by step parity
  double *bsum;           // [P][r][nblk]   per-slab sums of p entering each step; -1 = not yet published
  void *F;                // [P][nblk][r][slab] history rows, fp64 or (fast mode) fp32
  double *L;              // [P][r][r] Cholesky factor of h(K_S,K_S), row-major, lower triangle
  int32_t *idx, *r_eff;
  int64_t n, npad;
  int P, nblk, r, dpad;
  double *mail;           // [P][mail_words(r, dpad)] pivot records of the resident loop (see rpnys_step, section 3)
  int pr0;                // first problem of this launch (resident loop: the problems run in groups)
  int absent;             // test hooks of the give-up paths.  1: every workgroup but slab 0 of a problem leaves at
                          // once; 2: the workgroup that has found the pivot leaves before handing its record over
};

// History loads are streaming: each entry is read once per step and the working set (hundreds of MB)
// exceeds every cache, so they are issued as non-temporal loads, which measurably raises the sustained
// HBM read rate on this part.
typedef double dbl2 __attribute__((ext_vector_type(2)));
typedef float flt2 __attribute__((ext_vector_type(2)));
typedef float flt4 __attribute__((ext_vector_type(4)));
template <int KPT, typename H>
struct HistVec;
template <>
struct HistVec<1, double> {
  double v[1];
  __device__ __forceinline__ void load(const double *p) { v[0] = __builtin_nontemporal_load(p); }
};
template <>
struct HistVec<2, double> {
  double v[2];
  __device__ __forceinline__ void load(const double *p) {
    const dbl2 x = __builtin_nontemporal_load(reinterpret_cast<const dbl2 *>(p));
    v[0] = x.x; v[1] = x.y;
  }
};
template <>
struct HistVec<1, float> {
  float v[1];
  __device__ __forceinline__ void load(const float *p) { v[0] = __builtin_nontemporal_load(p); }
};
template <>
struct HistVec<2, float> {
  float v[2];
  __device__ __forceinline__ void load(const float *p) {
    const flt2 x = __builtin_nontemporal_load(reinterpret_cast<const flt2 *>(p));
    v[0] = x.x; v[1] = x.y;
  }
};

// The packed features of a thread's KPT keys, kept in registers across steps by the persistent driver
// (NC chunks of 4 features; NC = 0: not kept, streamed from memory every step).
template <typename T, int KPT, int NC>
struct KeyRegs {
  float x[NC > 0 ? NC : 1][KPT][kChunk / (sizeof(T) == 2 ? 2 : 1)];   // bf16 pairs stay packed in one 32-bit lane
};
template <typename T, int KPT, int NC>
__device__ __forceinline__ void load_key_regs(KeyRegs<T, KPT, NC> &kr, const T *kp, int64_t npad, bool exists) {
  if constexpr (NC > 0) {
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      if (!exists) {                                           // a thread whose keys are all padding: nothing to read
#pragma unroll
        for (int k = 0; k < KPT; ++k)
#pragma unroll
          for (int e = 0; e < (int)(sizeof(kr.x[0][0]) / sizeof(float)); ++e) kr.x[c][k][e] = 0.0f;
      } else if constexpr (sizeof(T) == 2) {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(kp + (size_t)c * npad * kChunk);
#pragma unroll
        for (int k = 0; k < KPT; ++k) {
          kr.x[c][k][0] = __uint_as_float(src[2 * k]);
          kr.x[c][k][1] = __uint_as_float(src[2 * k + 1]);
        }
      } else {
        float x[KPT][kChunk];
        load_chunk<T, KPT>(kp + (size_t)c * npad * kChunk, x);
#pragma unroll
        for (int k = 0; k < KPT; ++k)
#pragma unroll
          for (int e = 0; e < kChunk; ++e) kr.x[c][k][e] = x[k][e];
      }
    }
  }
}
template <typename T, int KPT, int NC>
__device__ __forceinline__ void key_chunk(const KeyRegs<T, KPT, NC> &kr, int c, float (&x)[KPT][kChunk]) {
#pragma unroll
  for (int k = 0; k < KPT; ++k) {
    if constexpr (sizeof(T) == 2) {
      const uint32_t lo = __float_as_uint(kr.x[c][k][0]), hi = __float_as_uint(kr.x[c][k][1]);
      // Opaque to the optimiser on purpose: the widened values are loop-invariant across steps, and hoisting them
      // out of the step loop would need four times the registers of the packed form.  The unpacking instructions
      // themselves are the opaque statements (an empty statement on a copy of the packed word would cost a move).
      uint32_t u0, u1, u2, u3;
      asm volatile("v_lshlrev_b32 %0, 16, %1" : "=v"(u0) : "v"(lo));
      asm volatile("v_and_b32 %0, 0xffff0000, %1" : "=v"(u1) : "v"(lo));
      asm volatile("v_lshlrev_b32 %0, 16, %1" : "=v"(u2) : "v"(hi));
      asm volatile("v_and_b32 %0, 0xffff0000, %1" : "=v"(u3) : "v"(hi));
      x[k][0] = __uint_as_float(u0); x[k][1] = __uint_as_float(u1);
      x[k][2] = __uint_as_float(u2); x[k][3] = __uint_as_float(u3);
    } else {
#pragma unroll
      for (int e = 0; e < kChunk; ++e) {
        float v = kr.x[c][k][e];
        asm volatile("" : "+v"(v));          // keeps the fp64 widening inside the step (see above)
        x[k][e] = v;
      }
    }
  }
}

// Device-coherent accesses for the few values one workgroup writes and another reads within the persistent
// launch (slab sums, pivot records, history rows): such stores are written through to memory and such loads bypass the
// non-coherent caches, so no cache-wide write-back or invalidate is needed between steps.
__device__ __forceinline__ void st_dev(double *p, double v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double ld_dev(const double *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_dev(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

struct StepShared {
  double sm[kThreads / kWave];
  int smi[kThreads / kWave];
  double s_base, s_ps, s_cb;
};

// Returns 1 after a step, 0 (state untouched) when the residual mass is exhausted, -1 if a bounded wait for another
// workgroup's slab sum ran out (POLL only).
// pown / flo: residual diagonal and floor of this thread's keys (registers); on return pown is updated.
// H = storage type of the history rows: double (pivots identical to a float64 reference) or float (fast mode: half
// the bytes; the row is rounded to fp32 BEFORE it enters the residual update, so the factorisation stays consistent
// with what later steps read back).
// SOLO: the problem has a single slab (small bins), so this workgroup is alone with it: the total mass is carried
// from step to step in `carry`, the residual diagonal is searched in registers, and nothing is polled, published or
// written for other workgroups (the history rows still go to memory: the Gram pass reads them).  The step's uniform
// and beta / tau^2 arrive as arguments (u_solo, bt_solo): the caller (k_rpnys_solo) has just computed them itself.
// LEAN: for loops of a few steps (bins of small rank), where the history stream is nothing and the registers are
// better spent on occupancy: one history row in flight instead of eight or twelve, none requested early, the pivot's
// features not read ahead.
template <typename T, int KPT, int NC, bool POLL, typename H, bool SOLO = false, bool LEAN = false, bool HANDOVER = true>
__device__ __forceinline__ int rpnys_step(const StepArgs &a, int i, int b, int pr, double *g, double *ksc,
                                          StepShared &sh, const KeyRegs<T, KPT, NC> &kr, double (&pown)[KPT],
                                          const double (&flo)[KPT], int *error, long long spin_limit, int hcn,
                                          double *carry = nullptr, double u_solo = 0.0, double bt_solo = 0.0) {
  constexpr int SLAB = kThreads * KPT;
  const int t = threadIdx.x;
  const int lane = t & (kWave - 1);
  const int rd = i & 1, wr = rd ^ 1;
  H *hc = reinterpret_cast<H *>(g + ((a.r + a.dpad + 1) & ~1));  // history cache [hcn][SLAB] behind g and ksc in LDS
  const double *bs = a.bsum + ((size_t)pr * a.r + i) * a.nblk;
  double *bs_next = a.bsum + ((size_t)pr * a.r + i + 1) * a.nblk;     // written only if i + 1 < r
  const double *pin = a.p + ((size_t)rd * a.P + pr) * a.npad;
  double *pout = a.p + ((size_t)wr * a.P + pr) * a.npad;
  H *Fb = reinterpret_cast<H *>(a.F) + ((size_t)pr * a.nblk + b) * a.r * SLAB;
  const int l_loc = t * KPT;
  const int64_t l_glob = (int64_t)b * SLAB + l_loc;

  // ---- 0. (single-launch loop) the first history rows of section 5 are requested now: which rows a step reads does
  // not depend on the pivot, only their weights g do, so these loads fly while the pivot is searched and a workgroup
  // keeps its share of the memory system busy during the part of the step that moves no data. ------------------------
  // Rows in flight per thread: eight 16-byte loads with two keys per thread, twelve narrower ones with one key
  // (those workgroups are small and few, and eight 8-byte loads each would not keep the memory system busy).
  constexpr int U = LEAN ? 1 : (KPT == 1 ? 12 : 8);
  constexpr bool EARLY = POLL && !SOLO && !LEAN;
  HistVec<KPT, H> early[EARLY ? U : 1];
  bool have_early = false;
  if constexpr (EARLY) {
    const int nc0 = i < hcn ? i : hcn;
    if (i - nc0 >= U) {
      const bool down0 = (i & 1) != 0;
      const ptrdiff_t fstep0 = down0 ? -(ptrdiff_t)SLAB : (ptrdiff_t)SLAB;
      const H *fp0 = Fb + l_loc + (size_t)(down0 ? i - 1 : nc0) * SLAB;
#pragma unroll
      for (int q = 0; q < U; ++q) early[q].load(fp0 + q * fstep0);
      have_early = true;
    }
  }

  // ---- 1. total mass = sum p (from the per-slab sums, in slab order) ----------------------------
  const int per = (a.nblk + kThreads - 1) / kThreads;
  const int e0 = t * per < a.nblk ? t * per : a.nblk;
  const int e1 = e0 + per < a.nblk ? e0 + per : a.nblk;
  double loc = 0.0;
  if constexpr (SOLO) {
    // nothing to collect
  } else if constexpr (POLL) {
    // The slab sums double as arrival flags: a slot holds -1 until its workgroup has finished the previous step
    // (whatever else the others need of that step travels in the pivot's record, section 3), so polling them is
    // the synchronisation between steps, and the successful poll already has the values.  Bounded: gives up after
    // spin_limit rounds, or when another workgroup has (the error word is looked at on every sixteenth round only:
    // its load is a trip through memory of its own).  The two barriers of a round also pace the polling: waves that
    // poll on their own, without them, were measured to slow the whole loop down by 5 % (they crowd the very cache
    // lines the awaited stores go to).
    long long spins = 0;
    while (true) {
      int ok = 1;
      loc = 0.0;
      for (int e = e0; e < e1; ++e) {
        const double v = ld_dev(bs + e);
        ok &= v >= 0.0;
        loc += v;
      }
      if (__syncthreads_and(ok)) break;
      if (++spins > spin_limit ||
          ((spins & 15) == 0 && __hip_atomic_load(error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
        if (t == 0) __hip_atomic_store(error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        spins = -1;
      }
      if (__syncthreads_or(spins < 0)) return -1;
      __builtin_amdgcn_s_sleep(1);
    }
  } else {
    for (int e = e0; e < e1; ++e) loc += ld_dev(bs + e);
  }
  double mass, inc = 0.0, excl = 0.0;
  if constexpr (SOLO) {
    mass = *carry;
  } else {
    inc = block_incl_scan(loc, sh.sm, &mass);
    excl = dpp_move<kDppWaveShr1>(0.0, inc);       // exclusive prefix = inclusive prefix of thread t-1
    if (lane == 0) {
      excl = 0.0;
      for (int k = 0; k < t / kWave; ++k) excl += sh.sm[k];
    }
  }
  if (!(mass > 0.0)) return 0;                     // h(K,K) is reproduced exactly by the pivots so far

  // ---- 2. the slab holding the draw: first slab whose inclusive prefix exceeds u * mass ----------------------
  double target = (SOLO ? u_solo : a.u[(size_t)pr * a.r + i]) * mass;
  int cand = INT_MAX;
  double cand_base = 0.0;
  int last_pos = -1;
  int bstar = 0;
  double base = 0.0;
  if constexpr (!SOLO) {
    {
      double run = excl;
      for (int e = e0; e < e1; ++e) {
        const double v = ld_dev(bs + e), nxt = run + v;
        if (nxt > target && cand == INT_MAX) { cand = e; cand_base = run; }
        if (v > 0.0) last_pos = e;
        run = nxt;
      }
    }
    bstar = block_reduce<int>(cand, sh.smi, MinOp());
    if (bstar == INT_MAX) {
      // Rounding left no slab above u * mass (u within an ulp of 1): take the last index of positive mass.
      bstar = block_reduce<int>(last_pos, sh.smi, MaxOp());
      target = INFINITY;
      if (t == 0) sh.s_base = 0.0;
    } else if (cand == bstar) {
      sh.s_base = cand_base;
    }
    __syncthreads();
    base = sh.s_base;
    bstar = bstar < 0 ? 0 : (bstar >= a.nblk ? a.nblk - 1 : bstar);   // only non-finite input can get here
  }

  // ---- 3. the pivot: its index inside that slab, its history column g_j = F_j(s) and k_s - kbar ---------------
  // Resident loop (RECORD): only the workgroup of slab bstar searches -- the slab's residual diagonal is in its own
  // registers, the first hcn history rows in its LDS -- and it leaves the pivot's record in memory for the other
  // slabs of the problem, which wait for it instead of repeating the search: nobody reads another slab's p or
  // history, so p never goes to memory and a step is published without waiting for its stores to complete
  // (measured on 512-step loops of 64 slabs: 2 us per step).  Not in the LEAN form and not for problems of a few
  // slabs (HANDOVER false, chosen by the host): there every slab searching for itself, all at once, was measured
  // faster than all but one waiting for that one (1 us per step with 8 slabs, 0.8 with 4, 0.2 with 16).
  constexpr bool RECORD = POLL && !LEAN && HANDOVER;
  const int nc = a.dpad / kChunk;
  const T *Kp = reinterpret_cast<const T *>(a.Kp) + (size_t)pr * nc * a.npad * kChunk;
  int64_t s_glob = -1;
  double cb;
  if (RECORD && b != bstar) {
    const double *rec = a.mail + (size_t)pr * mail_words(a.r, a.dpad) + mail_offset(i, a.dpad);
    const int nw = i + a.dpad + 2;
    long long spins = 0;
    while (true) {
      int ok = 1;
      for (int w = t; w < nw; w += kThreads) {
        const double v = ld_dev(rec + w);
        ok &= __double_as_longlong(v) != kMailEmpty;
        if (w < i) g[w] = v;
        else if (w < i + a.dpad) ksc[w - i] = v;
        else if (w == i + a.dpad) sh.s_ps = v;
        else sh.s_cb = v;
      }
      if (__syncthreads_and(ok)) break;                      // also publishes g, ksc, s_ps, s_cb to the workgroup
      if (++spins > spin_limit ||
          ((spins & 15) == 0 && __hip_atomic_load(error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))) {
        if (t == 0) __hip_atomic_store(error, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        spins = -1;
      }
      if (__syncthreads_or(spins < 0)) return -1;
      __builtin_amdgcn_s_sleep(1);
    }
    cb = sh.s_cb;
  } else {
    // (resident loop) rows of this slab's history beyond the LDS cache are read back from memory below, by other
    // threads than wrote them: every thread's stores of the earlier steps have completed before the barriers of
    // the scan that follows
    if constexpr (RECORD) __builtin_amdgcn_s_waitcnt(0x0F70);
    const double *ps = pin + (size_t)bstar * SLAB;
    double pv[KPT];
    loc = 0.0;
#pragma unroll
    for (int k = 0; k < KPT; ++k) { pv[k] = (SOLO || RECORD) ? pown[k] : ld_dev(ps + l_loc + k); loc += pv[k]; }
    double tot2;
    inc = block_incl_scan(loc, sh.sm, &tot2);
    excl = dpp_move<kDppWaveShr1>(0.0, inc);
    if (lane == 0) {
      excl = 0.0;
      for (int k = 0; k < t / kWave; ++k) excl += sh.sm[k];
    }
    cand = INT_MAX;
    last_pos = -1;
    {
      double run = base + excl;
#pragma unroll
      for (int k = 0; k < KPT; ++k) {
        const double nxt = run + pv[k];
        if (nxt > target && cand == INT_MAX) cand = l_loc + k;
        if (pv[k] > 0.0) last_pos = l_loc + k;
        run = nxt;
      }
    }
    int s_loc = block_reduce<int>(cand, sh.smi, MinOp());
    if (s_loc == INT_MAX) s_loc = block_reduce<int>(last_pos, sh.smi, MaxOp());
    if (s_loc < 0) s_loc = 0;                                          // non-finite input only
    if (s_loc / KPT == t) sh.s_ps = pv[s_loc % KPT];
    s_glob = (int64_t)bstar * SLAB + s_loc;

    const H *Fs = reinterpret_cast<const H *>(a.F) + ((size_t)pr * a.nblk + bstar) * a.r * SLAB + s_loc;
    for (int j = t; j < i; j += kThreads)
      g[j] = (SOLO || RECORD) && j < hcn ? (double)hc[(size_t)j * SLAB + s_loc] : (double)ld_dev(Fs + (size_t)j * SLAB);
    double cbp = 0.0;
    if (t < a.dpad) {
      const double kb = a.kbar[(size_t)pr * a.dpad + t];
      const double v = (double)to_float(Kp[((size_t)(t / kChunk) * a.npad + s_glob) * kChunk + (t % kChunk)]) - kb;
      ksc[t] = v;
      cbp = kb * v;
    }
    cb = block_sum(cbp, sh.sm);                    // <kbar, k_s - kbar>; also publishes g, ksc, s_ps
    if constexpr (RECORD) {
      if (a.absent == 2) return -1;                // (test hook) the others wait for a record that never comes
      double *rec = a.mail + (size_t)pr * mail_words(a.r, a.dpad) + mail_offset(i, a.dpad);
      const int nw = i + a.dpad + 2;
      for (int w = t; w < nw; w += kThreads)
        st_dev(rec + w, w < i ? g[w] : w < i + a.dpad ? ksc[w - i] : w == i + a.dpad ? sh.s_ps : cb);
    }
  }
  const double inv = 1.0 / sqrt(sh.s_ps);
  const double beta_tau = SOLO ? bt_solo : a.scal[(size_t)pr * 8 + 2];

  // ---- 5. history product  acc_l = sum_{j<i} F_j(l) g_j  (the O(n i) stream) ---------------------------
  // Rows are added in ascending order on even steps and in descending order on odd steps: the rows a step reads
  // last from memory are the rows the next step reads first, so whatever part of the history the memory-side
  // cache still holds is reused before it is evicted.  The order is fixed per step and does not depend on how
  // the loop is launched, so every launch form gives the same bits.
  // The first hcn rows of this slab's history are also kept in LDS (`hc`, single-launch forms only): they are
  // the rows every later step needs, so serving them from LDS removes about 2 hcn / r of the stream.  They take
  // their place in the same order: first on even steps, last on odd ones.
  double acc[KPT];
#pragma unroll
  for (int k = 0; k < KPT; ++k) acc[k] = 0.0;
  {
    const bool down = (i & 1) != 0;
    const int nc_rows = i < hcn ? i : hcn;                   // rows [0, nc_rows) come from LDS
    const int nh = i - nc_rows;                              // rows [nc_rows, i) from memory
    if (!down) {
      for (int j = 0; j < nc_rows; ++j) {
        const double gj = g[j];
#pragma unroll
        for (int k = 0; k < KPT; ++k) acc[k] = fma((double)hc[(size_t)j * SLAB + l_loc + k], gj, acc[k]);
      }
    }
    const ptrdiff_t fstep = down ? -(ptrdiff_t)SLAB : (ptrdiff_t)SLAB;
    const int gstep = down ? -1 : 1;
    const H *fp = Fb + l_loc + (size_t)(down ? i - 1 : nc_rows) * SLAB;
    const double *gp = g + (down ? i - 1 : nc_rows);
    int j = 0;
    if constexpr (EARLY) {
      if (have_early) {                                       // the batch requested in section 0
#pragma unroll
        for (int q = 0; q < U; ++q) {
          const double gj = gp[q * gstep];
#pragma unroll
          for (int k = 0; k < KPT; ++k) acc[k] = fma((double)early[q].v[k], gj, acc[k]);
        }
        fp += U * fstep;
        gp += U * gstep;
        j = U;
      }
    }
    for (; j + U <= nh; j += U) {
      HistVec<KPT, H> h[U];
#pragma unroll
      for (int q = 0; q < U; ++q) h[q].load(fp + q * fstep);
#pragma unroll
      for (int q = 0; q < U; ++q) {
        const double gj = gp[q * gstep];
#pragma unroll
        for (int k = 0; k < KPT; ++k) acc[k] = fma((double)h[q].v[k], gj, acc[k]);
      }
      fp += U * fstep;
      gp += U * gstep;
    }
    for (; j < nh; ++j) {
      HistVec<KPT, H> h;
      h.load(fp);
      const double gj = *gp;
#pragma unroll
      for (int k = 0; k < KPT; ++k) acc[k] = fma((double)h.v[k], gj, acc[k]);
      fp += fstep;
      gp += gstep;
    }
    if (down) {
      for (int j2 = nc_rows - 1; j2 >= 0; --j2) {
        const double gj = g[j2];
#pragma unroll
        for (int k = 0; k < KPT; ++k) acc[k] = fma((double)hc[(size_t)j2 * SLAB + l_loc + k], gj, acc[k]);
      }
    }
  }

  // ---- 6. kernel column  c_l = exp(beta_tau <k_l - kbar, k_s - kbar>)  (the O(n d) stream, or registers) --------
  double dot[KPT];
#pragma unroll
  for (int k = 0; k < KPT; ++k) dot[k] = 0.0;
  if constexpr (NC > 0) {
    // The pivot's features for chunk c + 1 are read from LDS before chunk c is worked on (the statement that keeps the
    // widening of the keys inside the step also keeps the compiler from moving LDS reads across it, so left alone
    // every chunk would start by waiting out an LDS round trip).
    double ks_next[kChunk];
#pragma unroll
    for (int e = 0; e < kChunk; ++e) ks_next[e] = ksc[e];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
      double ks[kChunk];
#pragma unroll
      for (int e = 0; e < kChunk; ++e) ks[e] = ks_next[e];
      if (c + 1 < NC && !LEAN) {
#pragma unroll
        for (int e = 0; e < kChunk; ++e) ks_next[e] = ksc[(c + 1) * kChunk + e];
      }
      if constexpr (LEAN) {                                    // (no registers to spare for reading ahead: every
        if (c > 0) {                                           // spilled register costs more than the LDS round trip)
#pragma unroll
          for (int e = 0; e < kChunk; ++e) ks[e] = ksc[c * kChunk + e];
        }
      }
      float x[KPT][kChunk];
      key_chunk<T, KPT, NC>(kr, c, x);
#pragma unroll
      for (int e = 0; e < kChunk; ++e) {
#pragma unroll
        for (int k = 0; k < KPT; ++k) dot[k] = fma((double)x[k][e], ks[e], dot[k]);
      }
    }
  } else {
    const T *kp = Kp + (size_t)l_glob * kChunk;
    const int nc_mine = l_glob < a.n ? nc : 0;                // a thread whose keys are all padding reads nothing
#pragma unroll 4
    for (int c = 0; c < nc_mine; ++c) {
      float x[KPT][kChunk];
      load_chunk<T, KPT>(kp + (size_t)c * a.npad * kChunk, x);
#pragma unroll
      for (int e = 0; e < kChunk; ++e) {
        const double ks = ksc[c * kChunk + e];
#pragma unroll
        for (int k = 0; k < KPT; ++k) dot[k] = fma((double)x[k][e], ks, dot[k]);
      }
    }
  }

  // ---- 7. new Cholesky row, residual diagonal, slab sum ------------------------------------------------
  double psum = 0.0;
  double fs = 0.0;
  bool own = false;
  double fkeep[KPT];
#pragma unroll
  for (int k = 0; k < KPT; ++k) {
    const int64_t l = l_glob + k;
    double f = (double)(H)((exp(beta_tau * (dot[k] - cb)) - acc[k]) * inv);     // as stored
    double pn = pown[k] - f * f;
    if (pn <= flo[k]) pn = 0.0;                                  // also clamps negatives (floor >= 0)
    if (l == s_glob) { pn = 0.0; fs = f; own = true; }
    if (l >= a.n) { pn = 0.0; f = 0.0; }
    st_dev(Fb + (size_t)i * SLAB + l_loc + k, (H)f);
    fkeep[k] = f;
    if constexpr (!SOLO && !(POLL && !LEAN && HANDOVER)) st_dev(pout + l, pn);   // (RECORD: nobody else reads it, see section 3)
    pown[k] = pn;
    psum += pn;
  }
  const double tot = block_sum(psum, sh.sm);
  if (i < hcn) {                                             // this thread's entries of the new row, for its own later reads
#pragma unroll
    for (int k = 0; k < KPT; ++k) hc[(size_t)i * SLAB + l_loc + k] = (H)fkeep[k];
  }
  if constexpr (SOLO) {
    *carry = tot;
    __syncthreads();                                         // the cached row is complete before the next step reads it
  } else {
    // (not RECORD: the other slabs read this one's p and history row, which must have completed: vmcnt(0))
    if constexpr (POLL && (LEAN || !HANDOVER)) __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();                                         // the cached row is complete before the next step reads it
    // Publishes the sum and, with it, the step.  RECORD: the other slabs need nothing else of this one: its history rows
    // are read back only by its own threads (section 5: each thread its own entries) and by its own search
    // (section 3, which waits for the stores first), and by the Gram pass after the launch.
    if (t == 0 && i + 1 < a.r) st_dev(bs_next + b, tot);
  }

  // ---- 8. bookkeeping by the slab that owns the pivot -----------------------------------------------------
  if (b == bstar) {
    double *Lr = a.L + ((size_t)pr * a.r + i) * a.r;
    for (int j = t; j < i; j += kThreads) Lr[j] = g[j];
    if (own) {
      Lr[i] = fs;
      a.idx[(size_t)pr * a.r + i] = (int32_t)s_glob;
    }
  }
  return 1;
}

// Driver 1: one launch per step; the kernel boundary is the synchronisation between steps.
template <typename T, int KPT, typename H>
__global__ __launch_bounds__(kThreads) void k_step(StepArgs a, int i) {
  extern __shared__ double dyn[];
  __shared__ StepShared sh;
  constexpr int SLAB = kThreads * KPT;
  const int t = threadIdx.x, b = blockIdx.x, pr = blockIdx.y;
  const int64_t l_glob = (int64_t)b * SLAB + t * KPT;
  const double *pin = a.p + ((size_t)(i & 1) * a.P + pr) * a.npad;
  double pown[KPT], flo[KPT];
#pragma unroll
  for (int k = 0; k < KPT; ++k) {
    pown[k] = pin[l_glob + k];
    flo[k] = a.floor[(size_t)pr * a.npad + l_glob + k];
  }
  KeyRegs<T, KPT, 0> none;
  if (rpnys_step<T, KPT, 0, false, H>(a, i, b, pr, dyn, dyn + a.r, sh, none, pown, flo, nullptr, 0, 0) == 0) {
    // Residual mass exhausted: carry the (all-zero) state into the other parity, leave row i of F zero, record
    // the number of pivots once.
    double *pout = a.p + ((size_t)((i & 1) ^ 1) * a.P + pr) * a.npad;
    H *Fb = reinterpret_cast<H *>(a.F) + ((size_t)pr * a.nblk + b) * a.r * SLAB;
#pragma unroll
    for (int k = 0; k < KPT; ++k) {
      pout[l_glob + k] = 0.0;
      Fb[(size_t)i * SLAB + t * KPT + k] = (H)0;
    }
    if (t == 0 && i + 1 < a.r) a.bsum[((size_t)pr * a.r + i + 1) * a.nblk + b] = 0.0;
    if (b == 0 && t == 0 && a.r_eff[pr] > i) a.r_eff[pr] = i;
  }
}

// Driver 2: the whole loop in one launch for the problems a.pr0 .. a.pr0 + gridDim.y - 1.  Requires all
// nblk * gridDim.y workgroups to fit on the device at once (the host sizes the groups against the kernel's occupancy).  The workgroups of one problem synchronise after every step through
// the slab sums themselves (see POLL above); the values that cross workgroups (slab sums, pivot records) are
// stored and loaded device-coherently (st_dev / ld_dev), so no cache-wide fence is needed.  Every wait is
// bounded: if a limit is hit (it never should be) the error word is set and every workgroup leaves.  With
// NC > 0 a thread keeps the packed features of its keys in registers for the whole loop, which removes the
// O(n d) key stream from every step.
// LEAN (see rpnys_step) fits the kernel with its keys in registers into 128 registers, i.e. four workgroups per
// compute unit: the many bins of a binned long sequence (a few steps each) are then all resident in one launch AND
// read their keys once instead of once per step.
template <typename T, int KPT, int NC, typename H, bool LEAN = false, bool HANDOVER = true>
__global__ __launch_bounds__(kThreads, (NC == 0 || LEAN) ? 4 : 2) void k_rpnys_persistent(StepArgs a, int *error, long long spin_limit,
                                                                  int hcn) {
  extern __shared__ double dyn[];
  __shared__ StepShared sh;
  constexpr int SLAB = kThreads * KPT;
  const int t = threadIdx.x, b = blockIdx.x, pr = a.pr0 + blockIdx.y;
  if (a.absent == 1 && b > 0) return;                        // (test hook) as if this workgroup never became resident
  const int64_t l_glob = (int64_t)b * SLAB + t * KPT;
  const int nc = a.dpad / kChunk;
  double pown[KPT], flo[KPT];
#pragma unroll
  for (int k = 0; k < KPT; ++k) {
    pown[k] = a.p[(size_t)pr * a.npad + l_glob + k];
    flo[k] = a.floor[(size_t)pr * a.npad + l_glob + k];
  }
  KeyRegs<T, KPT, NC> kr;
  load_key_regs<T, KPT, NC>(kr, reinterpret_cast<const T *>(a.Kp) + ((size_t)pr * nc * a.npad + l_glob) * kChunk,
                            a.npad, l_glob < a.n);
  int i = 0, rc = 1;
  for (; i < a.r; ++i) {
    rc = rpnys_step<T, KPT, NC, true, H, false, LEAN, HANDOVER>(a, i, b, pr, dyn, dyn + a.r, sh, kr, pown, flo, error, spin_limit, hcn);
    if (rc != 1) break;
  }
  if (rc == 0) {
    // Exhausted at step i (every workgroup of the problem sees the same sums and leaves at the same step):
    // rows i.. of this slab's history are zero for the Gram pass.
    H *Fb = reinterpret_cast<H *>(a.F) + ((size_t)pr * a.nblk + b) * a.r * SLAB;
    for (int j = i; j < a.r; ++j)
#pragma unroll
      for (int k = 0; k < KPT; ++k) Fb[(size_t)j * SLAB + t * KPT + k] = (H)0;
    if (b == 0 && t == 0) a.r_eff[pr] = i;
  }
}

// Driver 3: problems of a single slab (small bins: the image-model layer shapes, many bins of a long sequence).  One
// workgroup is alone with its problem, so the whole of Alg. 2's bin body up to the pivots runs here in one launch:
// ||k_l - kbar||^2 and R_K (what k_sqnorm computes, in the same order), the temperature, p_l = exp(beta_tau ||.||^2)
// and its floor (k_init_p), then the r steps in their SOLO form.  The residual diagonal, its floor and the total mass
// live in registers throughout; only the history rows, L, idx, r_eff and tau leave the workgroup.  grid (1, P); any
// number of workgroups may be resident (none waits for another).
struct SoloInit {
  const double *r_q;      // [P / bins]
  const double *u;        // [P][r] uniforms, or null: drawn from `seed` by the library's counter-based generator
  double *scal;           // [P][8]: 0 = R_K^2, 1 = tau, 2 = beta / tau^2, 3 = R_K
  double *tau_out;        // [P]
  unsigned long long seed;
  double rank_tol, tau_n, beta;
  int bins;
};

template <typename T, int KPT, int NC, typename H>
__global__ __launch_bounds__(kThreads, NC == 0 ? 4 : 2) void k_rpnys_solo(StepArgs a, SoloInit in, int hcn) {
  extern __shared__ double dyn[];
  __shared__ StepShared sh;
  constexpr int SLAB = kThreads * KPT;
  const int t = threadIdx.x, pr = blockIdx.y;
  const int64_t l_glob = t * KPT;
  const int nc = a.dpad / kChunk;
  double *skb = dyn + a.r;                                   // the step's k_s - kbar buffer is free until step 0
  if (t < a.dpad) skb[t] = a.kbar[(size_t)pr * a.dpad + t];
  const T *kp = reinterpret_cast<const T *>(a.Kp) + ((size_t)pr * nc * a.npad + l_glob) * kChunk;
  KeyRegs<T, KPT, NC> kr;
  load_key_regs<T, KPT, NC>(kr, kp, a.npad, l_glob < a.n);
  __syncthreads();

  double sq[KPT];
#pragma unroll
  for (int k = 0; k < KPT; ++k) sq[k] = 0.0;
  if (l_glob < a.n) {
    if constexpr (NC > 0) {
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        float x[KPT][kChunk];
        key_chunk<T, KPT, NC>(kr, c, x);
#pragma unroll
        for (int k = 0; k < KPT; ++k)
#pragma unroll
          for (int e = 0; e < kChunk; ++e) {
            const double df = (double)x[k][e] - skb[c * kChunk + e];
            sq[k] = fma(df, df, sq[k]);
          }
      }
    } else {
      for (int c = 0; c < nc; ++c) {
        float x[KPT][kChunk];
        load_chunk<T, KPT>(kp + (size_t)c * a.npad * kChunk, x);
#pragma unroll
        for (int k = 0; k < KPT; ++k)
#pragma unroll
          for (int e = 0; e < kChunk; ++e) {
            const double df = (double)x[k][e] - skb[c * kChunk + e];
            sq[k] = fma(df, df, sq[k]);
          }
      }
    }
  }
  double mx = 0.0;
#pragma unroll
  for (int k = 0; k < KPT; ++k) {
    if (l_glob + k >= a.n) sq[k] = 0.0;
    mx = fmax(mx, sq[k]);
  }
  mx = block_reduce<double>(mx, sh.sm, MaxOp());
  if (t == 0) {
    double tau, bt, rk;
    temperature(mx, in.r_q[pr / in.bins], in.tau_n, in.beta, &tau, &bt, &rk);
    sh.s_base = bt;
    in.scal[(size_t)pr * 8] = mx;
    in.scal[(size_t)pr * 8 + 1] = tau;
    in.scal[(size_t)pr * 8 + 2] = bt;
    in.scal[(size_t)pr * 8 + 3] = rk;
    in.tau_out[pr] = tau;
  }
  __syncthreads();
  const double beta_tau = sh.s_base;
  double pown[KPT], flo[KPT], s0 = 0.0;
#pragma unroll
  for (int k = 0; k < KPT; ++k) {
    const double v = (l_glob + k < a.n) ? exp(beta_tau * sq[k]) : 0.0;
    pown[k] = v;
    flo[k] = in.rank_tol * v;
    s0 += v;
  }
  double carry = block_sum(s0, sh.sm);

  int i = 0;
  for (; i < a.r; ++i) {
    const unsigned long long ctr = (unsigned long long)pr * a.r + i + 1ull;
    const double ui = in.u ? in.u[(size_t)pr * a.r + i]
                           : (double)(mix64(in.seed + ctr * 0x9E3779B97F4A7C15ull) >> 11) * 0x1.0p-53;
    if (rpnys_step<T, KPT, NC, false, H, true>(a, i, 0, pr, dyn, dyn + a.r, sh, kr, pown, flo, nullptr, 0, hcn, &carry,
                                               ui, beta_tau) != 1)
      break;
  }
  // Slots the loop did not fill (residual mass exhausted at step i): zero history rows for the Gram pass, idx = -1.
  H *Fb = reinterpret_cast<H *>(a.F) + (size_t)pr * a.r * SLAB;
  for (int j = i; j < a.r; ++j)
#pragma unroll
    for (int k = 0; k < KPT; ++k) Fb[(size_t)j * SLAB + t * KPT + k] = (H)0;
  for (int j = i + t; j < a.r; j += kThreads) a.idx[(size_t)pr * a.r + j] = -1;
  if (t == 0) a.r_eff[pr] = i;
}

// Driver 4: tiny problems (at most 128 keys and 16 pivots: the many-bin settings, where a layer has hundreds or
// thousands of them).  One WAVE per problem, four problems per workgroup: a lane keeps its one or two keys as floats
// in registers, the history rows of the problem sit in the wave's own piece of LDS, and every reduction, scan and
// broadcast of the step is a cross-lane operation, so the loop has no workgroup barrier and no memory round trip at
// all.  Same steps and the same arithmetic per key as the SOLO form above (sums over lanes associate differently:
// rounding only).  grid ceil(P / 4); dynamic LDS 4 x (DP doubles + r x 64 KW history entries).
__device__ __forceinline__ void wave_sync_lds() {            // LDS written by one lane is read by another lane next
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}
__device__ __forceinline__ double lane_value(double v, int lane) {      // lane: the same in every lane
  const long long b = __double_as_longlong(v);
  const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)b, lane);
  const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)((unsigned long long)b >> 32), lane);
  return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}
// Reductions over the wavefront, in every lane: a scan on data-parallel-primitive moves leaves the result in the last
// lane, from where it is read into a scalar register.
__device__ __forceinline__ double wave_sum(double v) { return lane_value(wave_incl_scan(v), kWave - 1); }
template <typename T, typename Op>
__device__ __forceinline__ T wave_reduce_idem(T v, Op op) {             // op(x, x) = x: minimum or maximum
  return wave_incl_scan_op(v, v, op);                                   // (the value itself as fill; result in lane 63)
}

template <typename T, int KW, int DP, typename H>
__global__ __launch_bounds__(kThreads, KW * DP <= 64 ? 2 : 1) void k_rpnys_wave(StepArgs a, SoloInit in) {
  extern __shared__ double dyn[];
  constexpr int NCH = DP / kChunk, ROW = kWave * KW;
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
  const int pr = blockIdx.x * (kThreads / kWave) + wv;
  if (pr >= a.P) return;                                     // no workgroup barrier below
  const int r = a.r;
  const size_t per_wave = (size_t)DP * sizeof(double) + (((size_t)r * ROW * sizeof(H) + 7) & ~(size_t)7);
  char *mine = reinterpret_cast<char *>(dyn) + wv * per_wave;
  double *skb = reinterpret_cast<double *>(mine);
  H *hist = reinterpret_cast<H *>(mine + (size_t)DP * sizeof(double));
  for (int c = lane; c < DP; c += kWave) skb[c] = a.kbar[(size_t)pr * DP + c];
  const int l0 = lane * KW;
  float x[KW][DP];
  {
    const T *kp = reinterpret_cast<const T *>(a.Kp) + ((size_t)pr * NCH * a.npad + l0) * kChunk;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      float xc[KW][kChunk];
      if (l0 < a.n) {
        load_chunk<T, KW>(kp + (size_t)c * a.npad * kChunk, xc);
      } else {
#pragma unroll
        for (int k = 0; k < KW; ++k)
#pragma unroll
          for (int e = 0; e < kChunk; ++e) xc[k][e] = 0.0f;
      }
#pragma unroll
      for (int k = 0; k < KW; ++k)
#pragma unroll
        for (int e = 0; e < kChunk; ++e) x[k][c * kChunk + e] = xc[k][e];
    }
  }
  wave_sync_lds();

  // ---- ||k_l - kbar||^2, R_K, temperature, p_0 ---------------------------------------------------------------
  double sq[KW], mx = 0.0;
#pragma unroll
  for (int k = 0; k < KW; ++k) sq[k] = 0.0;
#pragma unroll
  for (int c = 0; c < DP; ++c) {
    const double kb = skb[c];
#pragma unroll
    for (int k = 0; k < KW; ++k) {
      const double df = (double)x[k][c] - kb;
      sq[k] = fma(df, df, sq[k]);
    }
    if ((c & 7) == 7) __builtin_amdgcn_sched_barrier(0);
  }
#pragma unroll
  for (int k = 0; k < KW; ++k) {
    if (l0 + k >= a.n) sq[k] = 0.0;
    mx = fmax(mx, sq[k]);
  }
  mx = lane_value(wave_reduce_idem(mx, MaxOp()), kWave - 1);
  double tau, beta_tau, rk;
  temperature(mx, in.r_q[pr / in.bins], in.tau_n, in.beta, &tau, &beta_tau, &rk);   // every lane, same value
  if (lane == 0) {
    in.scal[(size_t)pr * 8] = mx;
    in.scal[(size_t)pr * 8 + 1] = tau;
    in.scal[(size_t)pr * 8 + 2] = beta_tau;
    in.scal[(size_t)pr * 8 + 3] = rk;
    in.tau_out[pr] = tau;
  }
  double p[KW], flo[KW], psum = 0.0;
#pragma unroll
  for (int k = 0; k < KW; ++k) {
    p[k] = (l0 + k < a.n) ? exp(beta_tau * sq[k]) : 0.0;
    flo[k] = in.rank_tol * p[k];
    psum += p[k];
  }
  double mass = wave_sum(psum);

  // ---- the r steps of Alg. 1 ---------------------------------------------------------------------------------
  H *Fb = reinterpret_cast<H *>(a.F) + (size_t)pr * r * a.npad;            // one slab per problem: rows of npad entries
  int i = 0;
  for (; i < r; ++i) {
    if (!(mass > 0.0)) break;
    // The keys stay as floats: without this the compiler keeps their fp64 widenings (loop invariants of the fully
    // unrolled products below) in registers as well, and spills.
#pragma unroll
    for (int k = 0; k < KW; ++k)
#pragma unroll
      for (int c = 0; c < DP; ++c) asm volatile("" : "+v"(x[k][c]));
    const double *kbar_lds = skb;                            // likewise kbar: read from LDS every step, not kept
    asm volatile("" : "+v"(kbar_lds));
    const unsigned long long ctr = (unsigned long long)pr * r + i + 1ull;
    const double ui = in.u ? in.u[(size_t)pr * r + i]
                           : (double)(mix64(in.seed + ctr * 0x9E3779B97F4A7C15ull) >> 11) * 0x1.0p-53;
    const double target = ui * mass;
    // the draw: first index whose inclusive prefix sum exceeds u * mass, else the last index of positive mass
    double loc = 0.0;
#pragma unroll
    for (int k = 0; k < KW; ++k) loc += p[k];
    const double inc = wave_incl_scan(loc);
    double run = dpp_move<kDppWaveShr1>(0.0, inc);           // exclusive prefix (lane 0: the fill, 0)
    int cand = INT_MAX, last_pos = -1;
#pragma unroll
    for (int k = 0; k < KW; ++k) {
      const double nxt = run + p[k];
      if (nxt > target && cand == INT_MAX) cand = l0 + k;
      if (p[k] > 0.0) last_pos = l0 + k;
      run = nxt;
    }
    cand = __builtin_amdgcn_readlane(wave_reduce_idem(cand, MinOp()), kWave - 1);
    last_pos = __builtin_amdgcn_readlane(wave_reduce_idem(last_pos, MaxOp()), kWave - 1);
    int s_loc = cand == INT_MAX ? last_pos : cand;
    if (s_loc < 0) s_loc = 0;                                // non-finite input only
    const int owner = s_loc / KW;
    const bool second = KW == 2 && (s_loc % KW) != 0;
    const double p_s0 = lane_value(p[0], owner), p_s1 = lane_value(p[KW - 1], owner);
    const double p_s = second ? p_s1 : p_s0;
    const double inv = 1.0 / sqrt(p_s);

    // kernel column: <k_l - kbar, k_s - kbar> = <k_l, k_s - kbar> - <kbar, k_s - kbar>
    double dot[KW], cb = 0.0;
#pragma unroll
    for (int k = 0; k < KW; ++k) dot[k] = 0.0;
#pragma unroll
    for (int c = 0; c < DP; ++c) {
      // (both keys of the owner lane are fetched and one is kept: selecting before the fetch would index x dynamically)
      float xs = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x[0][c]), owner));
      if constexpr (KW == 2) {
        const float xs1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x[KW - 1][c]), owner));
        xs = second ? xs1 : xs;
      }
      const double kb = kbar_lds[c];
      const double ks = (double)xs - kb;
      cb = fma(kb, ks, cb);
#pragma unroll
      for (int k = 0; k < KW; ++k) dot[k] = fma((double)x[k][c], ks, dot[k]);
      if ((c & 7) == 7) __builtin_amdgcn_sched_barrier(0);  // eight features at a time: keeps the widened values few
    }
    // history product  sum_{j<i} F_j(l) F_j(s)
    double acc[KW];
#pragma unroll
    for (int k = 0; k < KW; ++k) acc[k] = 0.0;
    for (int j = 0; j < i; ++j) {
      const double gj = (double)hist[(size_t)j * ROW + s_loc];
#pragma unroll
      for (int k = 0; k < KW; ++k) acc[k] = fma((double)hist[(size_t)j * ROW + l0 + k], gj, acc[k]);
    }
    // new Cholesky row and residual diagonal
    psum = 0.0;
#pragma unroll
    for (int k = 0; k < KW; ++k) {
      const int l = l0 + k;
      double f = (double)(H)((exp(beta_tau * (dot[k] - cb)) - acc[k]) * inv);
      double pn = p[k] - f * f;
      if (pn <= flo[k]) pn = 0.0;
      if (l == s_loc) {
        pn = 0.0;
        a.L[((size_t)pr * r + i) * r + i] = f;
        a.idx[(size_t)pr * r + i] = s_loc;
      }
      if (l >= a.n) { pn = 0.0; f = 0.0; }
      Fb[(size_t)i * a.npad + l] = (H)f;
      hist[(size_t)i * ROW + l] = (H)f;
      p[k] = pn;
      psum += pn;
    }
    if (lane < i) a.L[((size_t)pr * r + i) * r + lane] = (double)hist[(size_t)lane * ROW + s_loc];
    wave_sync_lds();                                         // row i is in LDS before the next step reads it
    mass = wave_sum(psum);
  }
  for (int j = i; j < r; ++j)
#pragma unroll
    for (int k = 0; k < KW; ++k) Fb[(size_t)j * a.npad + l0 + k] = (H)0;
  for (int j = i + lane; j < r; j += kWave) a.idx[(size_t)pr * r + j] = -1;
  if (lane == 0) a.r_eff[pr] = i;
}

// --------------------------------------------------------------------------------------------
// Gram pass  G = F [V, 1]  (Alg. 2 last line, reordered as in Sec. 2.1: weights times (V, 1_n) first).
// grid (nchunk * ncoltiles, ceil(r/128), P); workgroup tile = 128 rows of F x 16*CW value columns; thread
// (ty, tx) owns rows 8ty..8ty+7 and columns tx + 16 c: 8 x CW fp64 accumulators fed from LDS tiles of
// 16 keys (F as is, V widened to fp64 once per tile).  Partial sums per n-chunk, reduced in order later.
// --------------------------------------------------------------------------------------------
constexpr int kGramRows = 128, kGramKT = 16;

template <typename T, int CW, typename H>
__global__ __launch_bounds__(kThreads) void k_gram(const H *__restrict__ F, const T *__restrict__ V, int64_t n,
                                                   int nblk, int slab, int r, int dv, int slabs_per_chunk,
                                                   int nchunk, int ncoltiles, double *__restrict__ gpart) {
  __shared__ double Fs[kGramRows][kGramKT + 1];
  __shared__ double Vs[kGramKT][16 * CW];
  const int t = threadIdx.x, ch = blockIdx.x / ncoltiles, ct = blockIdx.x % ncoltiles, rt = blockIdx.y,
            pr = blockIdx.z;
  const int ty = t / 16, tx = t % 16;
  const int a0 = rt * kGramRows, col0 = ct * 16 * CW;
  double acc[8][CW];
  double rs[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    rs[q] = 0.0;
#pragma unroll
    for (int c = 0; c < CW; ++c) acc[q][c] = 0.0;
  }
  const int sb0 = ch * slabs_per_chunk;
  const int sb1 = sb0 + slabs_per_chunk < nblk ? sb0 + slabs_per_chunk : nblk;
  for (int sb = sb0; sb < sb1; ++sb) {
    const H *Fslab = F + ((size_t)pr * nblk + sb) * r * slab;
    for (int k0 = 0; k0 < slab; k0 += kGramKT) {
      const int64_t lbase = (int64_t)sb * slab + k0;
      if (lbase >= n) break;
      __syncthreads();
      {  // F tile: 128 rows x 16 keys; thread loads 8 consecutive keys of one row
        const int row = t / 2, seg = (t % 2) * 8;
        const bool ok = a0 + row < r;
        const H *src = Fslab + (size_t)(a0 + row) * slab + k0 + seg;
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          if constexpr (sizeof(H) == 8) {
            const double2 v = ok ? *reinterpret_cast<const double2 *>(src + e) : make_double2(0.0, 0.0);
            Fs[row][seg + e] = v.x;
            Fs[row][seg + e + 1] = v.y;
          } else {
            const float2 v = ok ? *reinterpret_cast<const float2 *>(src + e) : make_float2(0.f, 0.f);
            Fs[row][seg + e] = (double)v.x;
            Fs[row][seg + e + 1] = (double)v.y;
          }
        }
      }
      for (int e = t; e < kGramKT * 16 * CW; e += kThreads) {  // V tile: 16 keys x (16 CW) columns, as fp64
        const int kk = e / (16 * CW), c = e % (16 * CW);
        const int64_t l = lbase + kk;
        Vs[kk][c] = (l < n && col0 + c < dv) ? (double)to_float(V[((size_t)pr * n + l) * dv + col0 + c]) : 0.0;
      }
      __syncthreads();
#pragma unroll 2
      for (int kk = 0; kk < kGramKT; ++kk) {
        double fv[8], vv[CW];
#pragma unroll
        for (int q = 0; q < 8; ++q) fv[q] = Fs[8 * ty + q][kk];
#pragma unroll
        for (int c = 0; c < CW; ++c) vv[c] = Vs[kk][tx + 16 * c];
        if (tx == 0) {
#pragma unroll
          for (int q = 0; q < 8; ++q) rs[q] += fv[q];
        }
#pragma unroll
        for (int q = 0; q < 8; ++q)
#pragma unroll
          for (int c = 0; c < CW; ++c) acc[q][c] = fma(fv[q], vv[c], acc[q][c]);
      }
    }
  }
  const int dv1 = dv + 1;
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int arow = a0 + 8 * ty + q;
    if (arow >= r) continue;
    double *dst = gpart + (((size_t)pr * nchunk + ch) * r + arow) * dv1;
#pragma unroll
    for (int c = 0; c < CW; ++c)
      if (col0 + tx + 16 * c < dv) dst[col0 + tx + 16 * c] = acc[q][c];
    if (tx == 0 && ct == 0) dst[dv] = rs[q];
  }
}

// --------------------------------------------------------------------------------------------
// The same Gram pass on the fp64 matrix cores (v_mfma_f64_16x16x4_f64), for value widths of 64, 128 and 256: the
// pass is a dense fp64 contraction (2 n r (d_v + 1) flop against one read of F and V), bound by fp64 arithmetic,
// and the matrix pipe sustains its rate without the LDS tiles and register blocking the vector form needs.
// Lane (k = lane / 16, i = lane % 16) supplies A[i][k] = F_row(i)(key k) and B[k][j = i] = V(key k, column); the
// result tile holds D[4 v + lane / 16][lane % 16] in element v.  Column tile c of a lane covers value column
// NT (lane % 16) + c, so the NT values a lane needs from a key are adjacent in memory (one or two 16-byte loads) and
// its NT results of a row are adjacent in the output.  A wavefront owns 16 RT rows of F and all 16 NT columns; a
// workgroup 64 RT rows; the row sums (w = F 1) are added on the vector ALU from the same A operands.
// grid (nchunk, ceil(r / (64 RT)), P); same partial-sum layout as k_gram.
// --------------------------------------------------------------------------------------------
typedef double dbl4 __attribute__((ext_vector_type(4)));

template <typename T, int NT>
struct ValueRun {                                            // NT adjacent values of one row, in storage form
  static constexpr int WORDS = NT * (int)sizeof(T) / 4;
  uint32_t w[WORDS];
  __device__ __forceinline__ void zero() {
#pragma unroll
    for (int e = 0; e < WORDS; ++e) w[e] = 0u;
  }
  __device__ __forceinline__ void load(const T *__restrict__ src) {
    if constexpr (WORDS == 2) {
      const uint2 v = *reinterpret_cast<const uint2 *>(src);
      w[0] = v.x; w[1] = v.y;
    } else {
#pragma unroll
      for (int q = 0; q < WORDS / 4; ++q) {
        const uint4 v = reinterpret_cast<const uint4 *>(src)[q];
        w[4 * q] = v.x; w[4 * q + 1] = v.y; w[4 * q + 2] = v.z; w[4 * q + 3] = v.w;
      }
    }
  }
  __device__ __forceinline__ double get(int e) const {
    if constexpr (sizeof(T) == 4) return (double)__uint_as_float(w[e]);
    else return (double)__uint_as_float((e & 1) ? (w[e / 2] & 0xffff0000u) : (w[e / 2] << 16));
  }
};

template <typename T, int NT, typename H>
__global__ __launch_bounds__(kThreads, 2) void k_gram_mfma(const H *__restrict__ F, const T *__restrict__ V, int64_t n,
                                                        int nblk, int slab, int r, int slabs_per_chunk, int nchunk,
                                                        double *__restrict__ gpart) {
  constexpr int RT = NT <= 8 ? 2 : 1;                        // row tiles per wavefront: 16 RT x NT x 8 accumulator registers
  constexpr int U = (sizeof(T) == 4 && NT >= 8) ? 2 : 4;     // MFMA depth steps (4 keys each) per fetch, two fetches in flight
  constexpr int dv = 16 * NT;
  const int t = threadIdx.x, lane = t & (kWave - 1), wv = t / kWave;
  const int ch = blockIdx.x, pr = blockIdx.z;
  const int li = lane & 15, lk = lane >> 4;
  const int row_base = blockIdx.y * (64 * RT) + wv * (16 * RT);
  dbl4 acc[RT][NT];
  double rs[RT];
  bool rok[RT];
  size_t roff[RT];
#pragma unroll
  for (int q = 0; q < RT; ++q) {
    const int row = row_base + 16 * q + li;
    rok[q] = row < r;
    roff[q] = (size_t)(rok[q] ? row : 0) * slab;
    rs[q] = 0.0;
#pragma unroll
    for (int c = 0; c < NT; ++c) acc[q][c] = dbl4{0.0, 0.0, 0.0, 0.0};
  }
  // The chunk's keys [lbeg, lend) are walked in groups of 4 U (8 or 16; slabs are multiples of 16 keys, so a group lies in
  // one slab); the operands of the next group are fetched before the products of the current one are issued.
  const int sb0 = ch * slabs_per_chunk;
  const int sb1 = sb0 + slabs_per_chunk < nblk ? sb0 + slabs_per_chunk : nblk;
  const int64_t lbeg = (int64_t)sb0 * slab;
  const int64_t lend = (int64_t)sb1 * slab < n ? (int64_t)sb1 * slab : n;
  const H *Fp = F + (size_t)pr * nblk * r * slab;
  const T *Vp = V + (size_t)pr * n * dv + NT * li;
  auto fetch = [&](int64_t lg, double (&a)[U][RT], ValueRun<T, NT> (&b)[U]) {
    const int64_t sb = lg / slab;                            // uniform
    const H *Fs = Fp + (size_t)sb * r * slab + (lg - sb * slab);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t l = lg + 4 * u + lk;
      const bool kok = l < lend;
#pragma unroll
      for (int q = 0; q < RT; ++q) a[u][q] = (kok && rok[q]) ? (double)Fs[roff[q] + 4 * u + lk] : 0.0;
      if (kok) b[u].load(Vp + (size_t)l * dv);
      else b[u].zero();
    }
  };
  auto multiply = [&](const double (&a)[U][RT], const ValueRun<T, NT> (&b)[U]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
#pragma unroll
      for (int q = 0; q < RT; ++q) rs[q] += a[u][q];
#pragma unroll
      for (int c = 0; c < NT; ++c) {
        const double bv = b[u].get(c);
#pragma unroll
        for (int q = 0; q < RT; ++q) acc[q][c] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[u][q], bv, acc[q][c], 0, 0, 0);
      }
    }
  };
  if (lbeg < lend) {
    double a0[U][RT], a1[U][RT];
    ValueRun<T, NT> b0[U], b1[U];
    fetch(lbeg, a0, b0);
    for (int64_t lg = lbeg; lg < lend; lg += 8 * U) {
      fetch(lg + 4 * U, a1, b1);                             // past lend: zeros, nothing read
      multiply(a0, b0);
      fetch(lg + 8 * U, a0, b0);
      if (lg + 4 * U < lend) multiply(a1, b1);
    }
  }
  constexpr int dv1 = dv + 1;
  double *part = gpart + ((size_t)pr * nchunk + ch) * r * dv1;
#pragma unroll
  for (int q = 0; q < RT; ++q) {
    rs[q] += __shfl_xor(rs[q], 16, kWave);
    rs[q] += __shfl_xor(rs[q], 32, kWave);
    if (lk == 0 && rok[q]) part[(size_t)(row_base + 16 * q + li) * dv1 + dv] = rs[q];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int arow = row_base + 16 * q + 4 * v + lk;
      if (arow >= r) continue;
#pragma unroll
      for (int c = 0; c < NT; ++c) part[(size_t)arow * dv1 + NT * li + c] = acc[q][c][v];
    }
  }
}

// --------------------------------------------------------------------------------------------
// Gram pass for small ranks (r <= R <= 16; the binned regime of Sec. 2.5, where a bin gets a handful of pivots):
// the 128-row tiles above would be almost empty, and the pass is a pure stream over V.  Here a thread owns 4
// adjacent value columns of every (256 / tpr)-th key of the chunk and keeps R x 4 fp64 accumulators; tpr threads
// cover one value row with 8- or 16-byte loads, so a wavefront reads whole rows back to back.  The partial sums
// are combined in a fixed order (lane butterfly, then the four wavefronts in turn).
// grid (nchunk, 1, P); same partial-sum layout as k_gram.
// --------------------------------------------------------------------------------------------
// Four adjacent value columns of one row, kept in storage form until they are used (so that several rows can be
// in flight per thread without spending fp64 registers on them).  `vec`: rows are 4-element aligned.
template <typename T> struct Value4;
template <> struct Value4<float> {
  float4 raw;
  __device__ __forceinline__ void load(const float *__restrict__ row, int col, int dv, bool vec) {
    if (vec) raw = *reinterpret_cast<const float4 *>(row + col);
    else raw = make_float4(col < dv ? row[col] : 0.f, col + 1 < dv ? row[col + 1] : 0.f,
                           col + 2 < dv ? row[col + 2] : 0.f, col + 3 < dv ? row[col + 3] : 0.f);
  }
  __device__ __forceinline__ void widen(double (&v)[4]) const { v[0] = raw.x; v[1] = raw.y; v[2] = raw.z; v[3] = raw.w; }
};
template <> struct Value4<bf16_t> {
  uint2 raw;
  __device__ __forceinline__ void load(const bf16_t *__restrict__ row, int col, int dv, bool vec) {
    if (vec) {
      raw = *reinterpret_cast<const uint2 *>(row + col);
    } else {
      uint32_t e[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) e[c] = col + c < dv ? row[col + c].bits : 0u;
      raw = make_uint2(e[0] | (e[1] << 16), e[2] | (e[3] << 16));
    }
  }
  __device__ __forceinline__ void widen(double (&v)[4]) const {
    float x[kChunk];
    unpack_bf16x4(raw, x);
#pragma unroll
    for (int c = 0; c < 4; ++c) v[c] = (double)x[c];
  }
};

template <typename T, int R, typename H>
__global__ __launch_bounds__(kThreads) void k_gram_small(const H *__restrict__ F, const T *__restrict__ V,
                                                         int64_t n, int nblk, int slab, int r, int dv, int tpr,
                                                         int64_t chunk_keys, int nchunk,
                                                         double *__restrict__ gpart) {
  __shared__ double red[kThreads / kWave][kWave][5];
  const int t = threadIdx.x, ch = blockIdx.x, pr = blockIdx.z;
  const int lane = t & (kWave - 1), wv = t / kWave;
  const int kg = t / tpr, cg = t % tpr, kgs = kThreads / tpr;     // key group, column group, key groups
  const int col = 4 * cg;
  const bool active = col < dv;
  const bool vec = dv % 4 == 0;                                  // rows stay 4-element aligned
  double acc[R][4], rs[R];
#pragma unroll
  for (int j = 0; j < R; ++j) {
    rs[j] = 0.0;
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[j][c] = 0.0;
  }
  // The chunk's keys [lbeg, lend): whole slabs, or a piece of the only slab.
  const int64_t lbeg = (int64_t)ch * chunk_keys;
  const int64_t lend = lbeg + chunk_keys < n ? lbeg + chunk_keys : n;
  const T *Vp = V + (size_t)pr * n * dv;
  for (int sb = (int)(lbeg / slab); (int64_t)sb * slab < lend; ++sb) {
    const H *Fslab = F + ((size_t)pr * nblk + sb) * r * slab;
    constexpr int U = R <= 4 ? 4 : (R <= 8 ? 2 : 1);             // keys in flight per thread
    const int64_t s0 = (int64_t)sb * slab;
    const int kbeg = lbeg > s0 ? (int)(lbeg - s0) : 0;            // F is zero beyond n, V does not exist there
    const int kend = lend - s0 < slab ? (int)(lend - s0) : slab;
    for (int k0 = kbeg; k0 < kend; k0 += U * kgs) {
      Value4<T> raw[U];
      double f[U][R];
      bool ok[U];
#pragma unroll
      for (int q = 0; q < U; ++q) {
        const int l_loc = k0 + q * kgs + kg;
        const int64_t l = (int64_t)sb * slab + l_loc;
        ok[q] = active && l_loc < kend;
        const int l_safe = ok[q] ? l_loc : 0;
        raw[q].load(Vp + (size_t)(ok[q] ? l : 0) * dv, active ? col : 0, dv, vec);
#pragma unroll
        for (int j = 0; j < R; ++j) f[q][j] = (ok[q] && j < r) ? (double)Fslab[(size_t)j * slab + l_safe] : 0.0;
      }
#pragma unroll
      for (int q = 0; q < U; ++q) {
        double v[4];
        raw[q].widen(v);
        if (!ok[q]) v[0] = v[1] = v[2] = v[3] = 0.0;
#pragma unroll
        for (int j = 0; j < R; ++j) {
          rs[j] += f[q][j];
#pragma unroll
          for (int c = 0; c < 4; ++c) acc[j][c] = fma(f[q][j], v[c], acc[j][c]);
        }
      }
    }
  }
  const int dv1 = dv + 1;
#pragma unroll
  for (int j = 0; j < R; ++j) {
    double x[5] = {acc[j][0], acc[j][1], acc[j][2], acc[j][3], rs[j]};
    for (int off = tpr; off < kWave; off <<= 1)                   // key groups inside the wavefront
#pragma unroll
      for (int c = 0; c < 5; ++c) x[c] += __shfl_xor(x[c], off, kWave);
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 5; ++c) red[wv][lane][c] = x[c];
    __syncthreads();
    if (wv == 0 && lane < tpr && j < r) {
      double *dst = gpart + (((size_t)pr * nchunk + ch) * r + j) * dv1;
      double tot[5];
#pragma unroll
      for (int c = 0; c < 5; ++c) tot[c] = red[0][lane][c];
      for (int w2 = 1; w2 < kThreads / kWave; ++w2)
#pragma unroll
        for (int c = 0; c < 5; ++c) tot[c] += red[w2][lane][c];
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (col + c < dv) dst[col + c] = tot[c];
      if (lane == 0) dst[dv] = tot[4];
    }
  }
}

// The same pass for the common widths (d_v a multiple of 8, at most 512) and r <= 8, arranged for fewer and wider
// loads: a thread owns EIGHT value columns (one 16-byte load of a bf16 row) of four CONSECUTIVE keys at a time, so the
// four entries of a row of F it needs are adjacent in memory (two 16-byte loads instead of four 8-byte ones), and two
// such groups are in flight.  About a third of the load instructions per byte of k_gram_small.  Same partial-sum
// layout; the sums over key groups associate differently (rounding only).
template <typename T> struct Value8;
template <> struct Value8<float> {
  float4 a, b;
  __device__ __forceinline__ void load(const float *__restrict__ p) {
    a = reinterpret_cast<const float4 *>(p)[0];
    b = reinterpret_cast<const float4 *>(p)[1];
  }
  __device__ __forceinline__ void widen(double (&v)[8]) const {
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
};
template <> struct Value8<bf16_t> {
  uint4 raw;
  __device__ __forceinline__ void load(const bf16_t *__restrict__ p) { raw = *reinterpret_cast<const uint4 *>(p); }
  __device__ __forceinline__ void widen(double (&v)[8]) const {
    float x[kChunk], y[kChunk];
    unpack_bf16x4(make_uint2(raw.x, raw.y), x);
    unpack_bf16x4(make_uint2(raw.z, raw.w), y);
#pragma unroll
    for (int c = 0; c < 4; ++c) { v[c] = (double)x[c]; v[4 + c] = (double)y[c]; }
  }
};
template <typename H> struct Hist4;                            // four consecutive entries of a row of F
template <> struct Hist4<double> {
  dbl2 a, b;
  __device__ __forceinline__ void load(const double *p) {
    a = reinterpret_cast<const dbl2 *>(p)[0];
    b = reinterpret_cast<const dbl2 *>(p)[1];
  }
  __device__ __forceinline__ void zero() { a = dbl2{0.0, 0.0}; b = a; }
  __device__ __forceinline__ double at(int q) const { return q == 0 ? a.x : (q == 1 ? a.y : (q == 2 ? b.x : b.y)); }
};
template <> struct Hist4<float> {
  flt4 a;
  __device__ __forceinline__ void load(const float *p) { a = *reinterpret_cast<const flt4 *>(p); }
  __device__ __forceinline__ void zero() { a = flt4{0.f, 0.f, 0.f, 0.f}; }
  __device__ __forceinline__ double at(int q) const { return (double)a[q]; }
};

template <typename T, int R, typename H>
__global__ __launch_bounds__(kThreads) void k_gram_small8(const H *__restrict__ F, const T *__restrict__ V, int64_t n,
                                                          int nblk, int slab, int r, int dv, int tpr,
                                                          int64_t chunk_keys, int nchunk, double *__restrict__ gpart) {
  __shared__ double red[kThreads / kWave][kWave][9];
  const int t = threadIdx.x, ch = blockIdx.x, pr = blockIdx.z;
  const int lane = t & (kWave - 1), wv = t / kWave;
  const int kg = t / tpr, cg = t % tpr, kgs = kThreads / tpr;     // key group, column group (tpr = dv / 8), key groups
  const int col = 8 * cg;
  constexpr int G = 2;                                           // groups of four keys in flight per thread
  double acc[R][8], rs[R];
#pragma unroll
  for (int j = 0; j < R; ++j) {
    rs[j] = 0.0;
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[j][c] = 0.0;
  }
  // The chunk's keys [lbeg, lend): whole slabs, or a piece of the only slab; slabs and pieces are multiples of 64
  // keys, so a group of four keys never straddles either.  F is zero beyond n; V does not exist there.
  const int64_t lbeg = (int64_t)ch * chunk_keys;
  const int64_t lend = lbeg + chunk_keys < n ? lbeg + chunk_keys : n;
  const T *Vp = V + (size_t)pr * n * dv + col;
  const H *Fp = F + (size_t)pr * nblk * r * slab;
  for (int64_t l0 = lbeg + 4 * kg; l0 < lend; l0 += (int64_t)G * 4 * kgs) {
    Value8<T> raw[G][4];
    Hist4<H> f[G][R];
    bool ok[G][4];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const int64_t l = l0 + (int64_t)g * 4 * kgs;
      const bool any = l < lend;
      const int64_t ls = any ? l : lbeg;                          // (a key that exists: its loads are discarded)
      const int sb = (int)(ls / slab);
      const H *Fs = Fp + (size_t)sb * r * slab + (ls - (int64_t)sb * slab);
#pragma unroll
      for (int j = 0; j < R; ++j) {
        if (any && j < r) f[g][j].load(Fs + (size_t)j * slab);
        else f[g][j].zero();
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        ok[g][q] = l + q < lend;
        raw[g][q].load(Vp + (size_t)(ok[g][q] ? l + q : ls) * dv);
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        double v[8];
        raw[g][q].widen(v);
        if (!ok[g][q]) {
#pragma unroll
          for (int c = 0; c < 8; ++c) v[c] = 0.0;
        }
#pragma unroll
        for (int j = 0; j < R; ++j) {
          const double fj = ok[g][q] ? f[g][j].at(q) : 0.0;
          rs[j] += fj;
#pragma unroll
          for (int c = 0; c < 8; ++c) acc[j][c] = fma(fj, v[c], acc[j][c]);
        }
      }
  }
  const int dv1 = dv + 1;
#pragma unroll
  for (int j = 0; j < R; ++j) {
    double x[9];
#pragma unroll
    for (int c = 0; c < 8; ++c) x[c] = acc[j][c];
    x[8] = rs[j];
    for (int off = tpr; off < kWave; off <<= 1)                   // key groups inside the wavefront
#pragma unroll
      for (int c = 0; c < 9; ++c) x[c] += __shfl_xor(x[c], off, kWave);
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 9; ++c) red[wv][lane][c] = x[c];
    __syncthreads();
    if (wv == 0 && lane < tpr && j < r) {
      double *dst = gpart + (((size_t)pr * nchunk + ch) * r + j) * dv1;
      double tot[9];
#pragma unroll
      for (int c = 0; c < 9; ++c) tot[c] = red[0][lane][c];
      for (int w2 = 1; w2 < kThreads / kWave; ++w2)
#pragma unroll
        for (int c = 0; c < 9; ++c) tot[c] += red[w2][lane][c];
#pragma unroll
      for (int c = 0; c < 8; ++c) dst[col + c] = tot[c];
      if (lane == 0) dst[dv] = tot[8];
    }
  }
}

// Gram pass for small bins of small rank (one slab, at most 256 keys, r <= R <= 16: the image-model layer shapes and
// the many-bin settings).  There a problem is a few dozen keys, and what k_gram_small spends on adding up the partial
// sums of its threads exceeds the work.  Here a thread owns one value column of one piece of the bin's keys and all R
// rows of F: its R sums need no other thread; the row sums (w = F 1) are formed by every thread and written by the
// first.  tp threads (a power of two >= 64, >= d_v) cover a value row; a workgroup takes 256 / tp consecutive pieces,
// i.e. one run of keys, whose part of F it first copies to LDS with one coalesced pass: every lane of a wavefront
// needs the same entry of F, which LDS hands out as a broadcast, while as a per-lane load of one address it costs the
// memory pipeline some fifty clocks (and as a scalar load a round trip per handful of entries).
// grid (ceil(nchunk / (256 / tp)), 1, P); dynamic LDS R * (256 / tp) * chunk_keys doubles; same partial-sum layout as
// k_gram (one partial per piece).
template <typename T, int R, typename H>
__global__ __launch_bounds__(kThreads) void k_gram_cols(const H *__restrict__ F, const T *__restrict__ V, int64_t n,
                                                        int slab, int r, int dv, int tp, int chunk_keys, int nchunk,
                                                        double *__restrict__ gpart) {
  extern __shared__ double fs[];                              // [R][run]: rows of F over this workgroup's run of keys
  const int t = threadIdx.x, pr = blockIdx.z;
  const int sub = kThreads / tp, run = sub * chunk_keys;
  const int64_t run0 = (int64_t)blockIdx.x * run;
  const H *Fp = F + (size_t)pr * r * slab;                   // one slab per problem
  for (int e = t; e < R * run; e += kThreads) {
    const int j = e / run, k = e % run;
    fs[e] = (j < r && run0 + k < n) ? (double)Fp[(size_t)j * slab + run0 + k] : 0.0;
  }
  __syncthreads();
  const int c = t % tp, q = t / tp, ch = blockIdx.x * sub + q;
  if (ch >= nchunk) return;
  const bool active = c < dv;
  const int64_t lbeg = run0 + (int64_t)q * chunk_keys;
  const int kcount = lbeg + chunk_keys < n ? chunk_keys : (int)(n - lbeg);      // >= 1: ch < nchunk
  const T *Vp = V + ((size_t)pr * n + lbeg) * dv + (active ? c : 0);
  const double *fq = fs + q * chunk_keys;
  double acc[R], rs[R];
#pragma unroll
  for (int j = 0; j < R; ++j) acc[j] = rs[j] = 0.0;
  for (int k0 = 0; k0 < kcount; k0 += 8) {                    // eight keys per round; chunk_keys is a multiple of 16
    float v[8];                                               // and F is zero in LDS past the end of the bin
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = to_float(Vp[(size_t)(k0 + u < kcount ? k0 + u : kcount - 1) * dv]);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const double vd = (double)v[u];
#pragma unroll
      for (int j = 0; j < R; ++j) {
        const double f = fq[j * run + k0 + u];
        acc[j] = fma(f, vd, acc[j]);
        rs[j] += f;
      }
    }
  }
  const int dv1 = dv + 1;
  double *dst = gpart + ((size_t)pr * nchunk + ch) * r * dv1;
#pragma unroll
  for (int j = 0; j < R; ++j) {
    if (j < r) {
      if (active) dst[(size_t)j * dv1 + c] = acc[j];          // (an inactive thread read column 0: harmless, not stored)
      if (c == 0) dst[(size_t)j * dv1 + dv] = rs[j];
    }
  }
}

// Gt[pr][c][a] = sum over chunks (in chunk order) of gpart[pr][chunk][a][c].  grid (ceil(r*dv1/256), P).
__global__ __launch_bounds__(kThreads) void k_gram_reduce(const double *__restrict__ gpart, int r, int dv1,
                                                          int nchunk, double *__restrict__ Gt) {
  const int pr = blockIdx.y;
  const int gid = blockIdx.x * kThreads + threadIdx.x;
  if (gid >= r * dv1) return;
  const int c = gid / r, arow = gid % r;
  double s = 0.0;
  for (int ch = 0; ch < nchunk; ++ch) s += gpart[(((size_t)pr * nchunk + ch) * r + arow) * dv1 + c];
  Gt[((size_t)pr * dv1 + c) * r + arow] = s;
}

// --------------------------------------------------------------------------------------------
// Core solve  X = L^-T G  (W [V,1] = L^-T F [V,1]): back substitution, kSolveCols right-hand-side columns per
// workgroup, the columns held in LDS.  Rows are taken in panels of 32 from the bottom:
//   1. the 32 x 32 diagonal block of L goes to LDS; each column is solved inside the panel by its own 32
//      lanes (lane b keeps entry b in a register, the pivot value travels by a lane broadcast);
//   2. the panel's solution is eliminated from all rows above with one pass over the panel's rows of L
//      (contiguous in k, all threads), which amortises the memory latency over 32 substitution steps.
// grid (ceil(dv1/kSolveCols), P), block 32*kSolveCols.  Writes V_S (columns < dv) and w (column dv) as
// fp32; rows >= r_eff are zero.  LDS: (kSolveCols * r + 32*33 + kSolveCols*32) doubles.
// --------------------------------------------------------------------------------------------
constexpr int kSolveCols = 8, kPanel = 32;

__global__ __launch_bounds__(kSolveCols * 32) void k_solve(const double *__restrict__ L,
                                                           const double *__restrict__ Gt,
                                                           const int32_t *__restrict__ r_eff, int r, int dv,
                                                           float *__restrict__ v_s, float *__restrict__ w) {
  extern __shared__ double dyn[];
  double *gc = dyn;                                   // [kSolveCols][r]
  double *ld = gc + (size_t)kSolveCols * r;           // [32][33] diagonal block (reciprocals on the diagonal)
  double *xs = ld + kPanel * (kPanel + 1);            // [kSolveCols][32] panel solution
  const int pr = blockIdx.y, t = threadIdx.x, grp = t / 32, q = t % 32, nt = kSolveCols * 32;
  const int dv1 = dv + 1, c0 = blockIdx.x * kSolveCols;
  const int ncol = min(kSolveCols, dv1 - c0);
  const int re = r_eff[pr];
  const double *Lp = L + (size_t)pr * r * r;
  for (int e = t; e < ncol * re; e += nt) {
    const int c = e / re, k = e % re;
    gc[(size_t)c * r + k] = Gt[((size_t)pr * dv1 + c0 + c) * r + k];
  }
  for (int j1 = re; j1 > 0; j1 -= kPanel) {
    const int j0 = j1 > kPanel ? j1 - kPanel : 0, np = j1 - j0;
    __syncthreads();
    for (int e = t; e < np * np; e += nt) {
      const int a = e / np, bcol = e % np;
      if (bcol <= a) {
        const double v = Lp[(size_t)(j0 + a) * r + j0 + bcol];
        ld[a * (kPanel + 1) + bcol] = bcol == a ? 1.0 / v : v;
      }
    }
    __syncthreads();
    if (grp < ncol) {                                  // 1. solve inside the panel: x_a = g_a / L_aa, g_b -= L_ab x_a
      double gb = q < np ? gc[(size_t)grp * r + j0 + q] : 0.0;
      double xb = 0.0;
      const bool upper = (t & 32) != 0;                 // this column's 32 lanes are the upper half of their wavefront
#pragma unroll
      for (int a = kPanel - 1; a >= 0; --a) {
        if (a >= np) continue;                            // uniform: only the topmost panel is short
        const double glo = lane_value(gb, a), ghi = lane_value(gb, a + 32);
        const double xa = (upper ? ghi : glo) * ld[a * (kPanel + 1) + a];
        if (q == a) xb = xa;
        if (q < a) gb = fma(-ld[a * (kPanel + 1) + q], xa, gb);
      }
      if (q < np) {
        gc[(size_t)grp * r + j0 + q] = xb;
        xs[grp * kPanel + q] = xb;
      }
    }
    __syncthreads();
    for (int k = t; k < j0; k += nt) {                 // 2. eliminate the panel from the rows above
      double upd[kSolveCols];
#pragma unroll
      for (int c = 0; c < kSolveCols; ++c) upd[c] = 0.0;
#pragma unroll 8
      for (int a = 0; a < np; ++a) {
        const double lv = Lp[(size_t)(j0 + a) * r + k];
#pragma unroll
        for (int c = 0; c < kSolveCols; ++c) upd[c] = fma(lv, xs[c * kPanel + a], upd[c]);
      }
#pragma unroll
      for (int c = 0; c < kSolveCols; ++c)
        if (c < ncol) gc[(size_t)c * r + k] -= upd[c];
    }
  }
  __syncthreads();
  for (int e = t; e < ncol * r; e += nt) {
    const int c = e / r, j = e % r;
    const float val = j < re ? (float)gc[(size_t)c * r + j] : 0.0f;
    if (c0 + c < dv) v_s[((size_t)pr * r + j) * dv + c0 + c] = val;
    else w[(size_t)pr * r + j] = val;
  }
}

// The same solve for small ranks (r <= kSolveSmall, i.e. binned problems with a handful of pivots each, of which there
// are many): one thread per (problem, right-hand-side column) substitutes backwards through its own copy of the
// column, in the order k_solve uses inside a panel (x_a = g_a * (1 / L_aa), then g_b -= L_ab x_a for b < a), so the
// two kernels give the same bits.  The right-hand side is summed here from the Gram pass's partial sums, in chunk order
// as k_gram_reduce does (adjacent threads read adjacent columns), which saves that launch.  grid ceil(P * (dv + 1) / 256).
constexpr int kSolveSmall = 16;

__global__ __launch_bounds__(kThreads) void k_solve_small(const double *__restrict__ L, const double *__restrict__ gpart,
                                                          int nchunk, const int32_t *__restrict__ r_eff, int P, int r,
                                                          int dv, float *__restrict__ v_s, float *__restrict__ w) {
  const int dv1 = dv + 1;
  const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (gid >= (int64_t)P * dv1) return;
  const int pr = (int)(gid / dv1), c = (int)(gid % dv1);
  const int re = min(r_eff[pr], r);
  const double *Lp = L + (size_t)pr * r * r;
  double g[kSolveSmall];
#pragma unroll
  for (int j = 0; j < kSolveSmall; ++j) g[j] = 0.0;
  int ch = 0;
  for (; ch + 2 <= nchunk; ch += 2) {                         // chunk order per entry; two chunks' loads in flight
    double x[2][kSolveSmall];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      const double *gp = gpart + ((size_t)pr * nchunk + ch + q) * r * dv1 + c;
#pragma unroll
      for (int j = 0; j < kSolveSmall; ++j) x[q][j] = j < re ? gp[(size_t)j * dv1] : 0.0;
    }
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int j = 0; j < kSolveSmall; ++j)
        if (j < re) g[j] += x[q][j];
  }
  for (; ch < nchunk; ++ch) {
    const double *gp = gpart + ((size_t)pr * nchunk + ch) * r * dv1 + c;
#pragma unroll
    for (int j = 0; j < kSolveSmall; ++j)
      if (j < re) g[j] += gp[(size_t)j * dv1];
  }
#pragma unroll
  for (int a = kSolveSmall - 1; a >= 0; --a) {
    if (a < re) {
      const double xa = g[a] * (1.0 / Lp[(size_t)a * r + a]);
      g[a] = xa;
#pragma unroll
      for (int b = 0; b < kSolveSmall; ++b)
        if (b < a) g[b] = fma(-Lp[(size_t)a * r + b], xa, g[b]);
    }
  }
#pragma unroll
  for (int j = 0; j < kSolveSmall; ++j) {
    if (j < r) {
      const float val = j < re ? (float)g[j] : 0.0f;
      if (c < dv) v_s[((size_t)pr * r + j) * dv + c] = val;
      else w[(size_t)pr * r + j] = val;
    }
  }
}

// K_S = original key rows at the pivots (Alg. 2: recentred pivots plus the mean), zero in unused slots.  Pivot indices
// were found relative to the bin; once the row is read, the slot's index is rewritten as an index into the head's
// n * bins keys.  grid (r, P), n = keys per bin.
// `error` (null unless the loop ran as resident launches): a wait inside the loop that ran out (never expected) is
// reported here, in the last launch of the pass, as r_eff = -1 for every problem.
template <typename T>
__global__ void k_gather(const T *__restrict__ K, int32_t *__restrict__ idx, int64_t n, int d, int r, int bins,
                         T *__restrict__ k_s, const int *__restrict__ error, int32_t *__restrict__ r_eff) {
  const int i = blockIdx.x, pr = blockIdx.y;
  if (error && i == 0 && threadIdx.x == 0 && *error) r_eff[pr] = -1;
  const int s = idx[(size_t)pr * r + i];
  for (int j = threadIdx.x; j < d; j += blockDim.x) {
    T z;
    from_float(0.0f, &z);
    k_s[((size_t)pr * r + i) * d + j] = s >= 0 ? K[((size_t)pr * n + s) * d + j] : z;
  }
  __syncthreads();                                       // every thread has read the local index
  if (threadIdx.x == 0 && bins > 1 && s >= 0) idx[(size_t)pr * r + i] = s + (int32_t)((pr % bins) * n);
}

// Debug / test output: the Nystrom weights themselves, W = h(K_S,K_S)^-1 h(K_S,K) = L^-T F (Alg. 1's return value;
// the pass itself only ever forms W V and W 1).  One thread per key solves L^T x = F(:, l) by back substitution, its
// unknowns kept in the output column it is writing (a thread reads back only what it wrote).  grid (ceil(n / 256), P);
// W is [P][r][n] with n the keys per bin; rows from r_eff on are zero.
template <typename H>
__global__ __launch_bounds__(kThreads) void k_debug_weights(const H *__restrict__ F, const double *__restrict__ L,
                                                            const int32_t *__restrict__ r_eff, int64_t n, int nblk,
                                                            int slab, int r, double *__restrict__ W) {
  const int pr = blockIdx.y;
  const int64_t l = (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (l >= n) return;
  int re = r_eff[pr];
  re = re < 0 ? 0 : (re > r ? r : re);
  const H *Fp = F + ((size_t)pr * nblk + l / slab) * r * slab + l % slab;        // row j: + j * slab
  const double *Lp = L + (size_t)pr * r * r;
  double *Wp = W + (size_t)pr * r * n + l;                                       // row j: + j * n
  for (int j = r - 1; j >= re; --j) Wp[(size_t)j * n] = 0.0;
  for (int j = re - 1; j >= 0; --j) {
    double acc = (double)Fp[(size_t)j * slab];
    for (int k = j + 1; k < re; ++k) acc -= Lp[(size_t)k * r + j] * Wp[(size_t)k * n];
    Wp[(size_t)j * n] = acc / Lp[(size_t)j * r + j];
  }
}

#define LAUNCH_CHECK()                                   \
  do {                                                   \
    if (hipGetLastError() != hipSuccess) return WILDCAT_EHIP; \
  } while (0)

// The launch form of the selection loop for this shape on the current device: the kernel (null: one launch per
// step), its dynamic LDS size and the number of history rows cached in LDS -- whatever LDS the compute unit has left
// once every workgroup it must hold has its share.
struct LoopPlan {
  LoopChoice c;
  const void *fn;
  size_t lds;
  int hcn;
};

constexpr int kWaveRank = 16;                                // k_rpnys_wave: at most this many pivots (lane j < i writes L)

template <typename T, typename H>
const void *wave_kernel(const Shape &s, int dpad) {
  if (s.r > kWaveRank) return nullptr;
  if (dpad == 64 && s.n <= 64) return (const void *)k_rpnys_wave<T, 1, 64, H>;
  if (dpad == 64 && s.n <= 128) return (const void *)k_rpnys_wave<T, 2, 64, H>;
  if (dpad == 128 && s.n <= 64) return (const void *)k_rpnys_wave<T, 1, 128, H>;
  return nullptr;
}

// The workgroup-per-slab loop kernel: `solo` = problems of one slab, `regs` = keys kept in registers (only where
// keys_fit_registers says so), nc = chunks of four features.
constexpr int kLeanRank = 16;                                // loops of at most this many steps take the LEAN kernels
constexpr int kHandoverSlabs = 24;                           // problems of at least this many slabs hand the pivot over (rpnys_step, section 3)

template <typename T, int KPT, int NC, typename H>
const void *resident_kernel(bool handover) {
  return handover ? (const void *)k_rpnys_persistent<T, KPT, NC, H, false, true>
                  : (const void *)k_rpnys_persistent<T, KPT, NC, H, false, false>;
}

template <typename T, int KPT, typename H>
const void *loop_kernel(bool solo, bool regs, int nc, bool lean = false, bool handover = true) {
  constexpr int regs_per_chunk = KPT * (sizeof(T) == 2 ? 2 : 4);
  if constexpr (16 * regs_per_chunk <= 64) {                  // (bf16, d <= 64: the keys take at most 64 registers)
    if (lean && regs && !solo && nc == 16) return (const void *)k_rpnys_persistent<T, KPT, 16, H, true>;
  }
  if constexpr (32 * regs_per_chunk <= 128) {
    if (regs && nc == 32) return solo ? (const void *)k_rpnys_solo<T, KPT, 32, H> : resident_kernel<T, KPT, 32, H>(handover);
  }
  if constexpr (16 * regs_per_chunk <= 128) {
    if (regs && nc == 16) return solo ? (const void *)k_rpnys_solo<T, KPT, 16, H> : resident_kernel<T, KPT, 16, H>(handover);
  }
  return solo ? (const void *)k_rpnys_solo<T, KPT, 0, H> : resident_kernel<T, KPT, 0, H>(handover);
}

inline size_t loop_base_lds(const Shape &s, const Plan &pl) { return (size_t)((s.r + pl.dpad + 1) & ~1) * sizeof(double); }

template <typename T, int KPT, typename H>
int device_caps(const Shape &s, const Plan &pl, DeviceCaps *caps) {
  const int nc = pl.dpad / kChunk;
  const bool solo = pl.nblk == 1;
  const size_t base = loop_base_lds(s, pl);
  caps->cus = compute_units();
  caps->occ_regs = caps->occ_stream = 0;
  if (keys_fit_registers(s.dtype, pl.kpt, pl.dpad) &&
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&caps->occ_regs, loop_kernel<T, KPT, H>(solo, true, nc, s.r <= kLeanRank,
                                                                                        pl.nblk >= kHandoverSlabs),
                                                   kThreads, base) != hipSuccess)
    caps->occ_regs = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&caps->occ_stream,
                                                   loop_kernel<T, KPT, H>(solo, false, nc, false, pl.nblk >= kHandoverSlabs), kThreads,
                                                   base) != hipSuccess)
    caps->occ_stream = 0;
  (void)hipGetLastError();                                   // a failed query must not be reported by a later launch check
  return WILDCAT_OK;
}

template <typename T, int KPT, typename H>
LoopPlan plan_loop(const Shape &s, const Plan &pl) {
  LoopPlan lp = {{kLoopSteps, 0, s.P, 1, 0}, nullptr, 0, 0};
  if (!pl.persistent || s.loop_driver == WILDCAT_LOOP_STEPS) return lp;
  DeviceCaps caps;
  device_caps<T, KPT, H>(s, pl, &caps);
  LoopChoice c = choose_loop(s, pl, caps);
  if (c.kind == kLoopWave) {
    const void *wfn = wave_kernel<T, H>(s, pl.dpad);
    const int kw = s.n <= 64 ? 1 : 2;
    const size_t per_wave = (size_t)pl.dpad * sizeof(double) + (((size_t)s.r * kWave * kw * sizeof(H) + 7) & ~(size_t)7);
    const size_t lds = per_wave * (kThreads / kWave);
    if (wfn && (lds <= 64 * 1024 ||
                hipFuncSetAttribute(wfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess)) {
      lp.c = c; lp.fn = wfn; lp.lds = lds;
      return lp;
    }
    c = choose_loop(s, pl, caps, false);                     // the wave form cannot run here: a workgroup per problem
  }
  if (c.kind == kLoopSteps) return lp;
  const bool solo = c.kind == kLoopSolo;
  const void *fn = loop_kernel<T, KPT, H>(solo, c.keys_in_regs != 0, pl.dpad / kChunk, s.r <= kLeanRank, pl.nblk >= kHandoverSlabs);
  const size_t base = loop_base_lds(s, pl);
  lp.c = c; lp.fn = fn; lp.lds = base;
  // History cache: optional, and only if the kernel stays resident with it.
  const int need = c.need > 0 ? c.need : 1;
  int dev = 0, lds_cu = 0;
  if (hipGetDevice(&dev) == hipSuccess &&
      hipDeviceGetAttribute(&lds_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) == hipSuccess && lds_cu > 0) {
    const int64_t share = (int64_t)lds_cu / need - 2048 - (int64_t)base;    // static LDS and allocation granules
    const int64_t row = (int64_t)kThreads * KPT * sizeof(H);
    int hcn = share > 0 ? (int)(share / row) : 0;
    if (hcn > s.r) hcn = s.r;
    if (hcn > 0) {
      const size_t lds = base + (size_t)hcn * row;
      int per_cu2 = 0;
      if ((lds <= 64 * 1024 ||
           hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess) &&
          hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu2, fn, kThreads, lds) == hipSuccess && per_cu2 >= need) {
        lp.lds = lds;
        lp.hcn = hcn;
      }
    }
  }
  (void)hipGetLastError();
  return lp;
}

// `s` is the bin view of the request (wildcat::bin_view): P problems = bins, n keys and r pivots per bin.
template <typename T, int KPT, typename H>
int run_compress(const Shape &s, const Plan &pl, const T *K, const T *V, const wildcat_opts *o, uint64_t seed,
                 wildcat_coreset *out) {
  char *ws = (char *)o->workspace;
  double *kbar = (double *)(ws + pl.off_kbar);
  T *Kp = (T *)(ws + pl.off_kp);
  double *d0 = (double *)(ws + pl.off_d0);
  double *p = (double *)(ws + pl.off_p);
  double *bsum = (double *)(ws + pl.off_bsum);
  double *scal = (double *)(ws + pl.off_scal);
  H *F = (H *)(ws + pl.off_F);
  double *L = (double *)(ws + pl.off_L);
  double *gpart = (double *)(ws + pl.off_gpart);
  double *Gt = (double *)(ws + pl.off_g);
  double *mpart = (double *)(ws + pl.off_mpart);
  float *vminpart = (float *)(ws + pl.off_vminpart);
  float *vmaxpart = (float *)(ws + pl.off_vmaxpart);
  double *u_gen = (double *)(ws + pl.off_u);
  hipStream_t st = s.stream;
  const int P = s.P;

  int lpr = 1;
  while (lpr < s.d || lpr < s.dv || lpr < pl.dpad) lpr <<= 1;
  const int nc = pl.dpad / kChunk;
  constexpr int epp = 16 / (int)sizeof(T);
  auto pow2_pieces = [](int width) {
    const int pieces = width / epp;
    return width % epp == 0 && pieces >= 1 && pieces <= kWave && (pieces & (pieces - 1)) == 0;
  };
  int nparts = pl.nb0;                                        // partial results per problem
  if (pow2_pieces(s.d) && pow2_pieces(s.dv)) {
    const int tk = s.d * (int)sizeof(T) <= 256 ? 64 : 32;     // tile height: at most 33 KB of LDS for the tile
    int64_t kpw = (pl.npad + pl.nb0 - 1) / pl.nb0;
    kpw = (kpw + tk - 1) / tk * tk;
    nparts = (int)((pl.npad + kpw - 1) / kpw);                // <= nb0
    const size_t lds = (size_t)tk * (s.d * sizeof(T) + 8);
    hipLaunchKernelGGL((k_pack_stats<T>), dim3(nparts, P), dim3(kThreads), lds, st, K, V, s.n, pl.npad, s.d, s.dv,
                       (int)kpw, tk, nparts, Kp, mpart, vminpart, vmaxpart);
    LAUNCH_CHECK();
  } else {
    hipLaunchKernelGGL((k_col_stats<T>), dim3(pl.nb0, P), dim3(kThreads), 0, st, K, V, s.n, s.d, s.dv, pl.dpad, pl.nb0,
                       lpr, mpart, vminpart, vmaxpart);
    LAUNCH_CHECK();
    const int64_t packs = (pl.npad * nc + kThreads - 1) / kThreads;
    hipLaunchKernelGGL((k_pack<T>), dim3((unsigned)packs, P), dim3(kThreads), 0, st, K, s.n, pl.npad, s.d, pl.dpad, Kp);
    LAUNCH_CHECK();
  }
  const int slices = lpr >= 64 ? 4 : 1;                       // (lpr is a power of two, at most kFinalThreads)
  hipLaunchKernelGGL(k_col_final, dim3(P / s.bins, slices), dim3(kFinalThreads / slices), 0, st, mpart, vminpart, vmaxpart,
                     s.n, s.dv, pl.dpad, nparts, s.bins, lpr, kbar, out->v_min, out->v_max, (unsigned long long *)scal);
  LAUNCH_CHECK();
  const LoopPlan lp = plan_loop<T, KPT, H>(s, pl);
  const bool one_slab_form = lp.c.kind == kLoopSolo || lp.c.kind == kLoopWave;   // these also do the work of k_sqnorm, k_init_p
  const double tau_n = (double)(s.tau_full_n ? s.n * s.bins : s.n);
  if (!one_slab_form) {
    hipLaunchKernelGGL((k_sqnorm<T, KPT>), dim3(pl.nblk, P), dim3(kThreads), 0, st, Kp, kbar, s.n, pl.npad, pl.dpad, d0,
                       (unsigned long long *)scal);
    LAUNCH_CHECK();
    hipLaunchKernelGGL((k_init_p<KPT>), dim3(pl.nblk, P), dim3(kThreads), 0, st, s.n, pl.npad, pl.nblk, s.r, s.rank_tol,
                       s.bins, tau_n, s.beta, o->r_q, scal, out->tau, d0, p, bsum, out->idx, out->r_eff,
                       o->uniforms ? (double *)nullptr : u_gen, (unsigned long long)seed, (int *)(ws + pl.off_sync),
                       lp.c.kind == kLoopResident && pl.nblk >= kHandoverSlabs ? (long long *)(ws + pl.off_mail)
                                                                              : (long long *)nullptr,
                       (long long)mail_words(s.r, pl.dpad));
    LAUNCH_CHECK();
  }

  StepArgs a;
  a.Kp = Kp; a.kbar = kbar; a.scal = scal; a.floor = d0; a.u = o->uniforms ? o->uniforms : u_gen;
  a.p = p; a.bsum = bsum; a.F = F; a.L = L; a.idx = out->idx; a.r_eff = out->r_eff;
  a.n = s.n; a.npad = pl.npad; a.P = P; a.nblk = pl.nblk; a.r = s.r; a.dpad = pl.dpad;
  a.pr0 = 0; a.absent = 0; a.mail = (double *)(ws + pl.off_mail);
  if (o->ev_loop_begin && hipEventRecord((hipEvent_t)o->ev_loop_begin, st) != hipSuccess) return WILDCAT_EHIP;
  const size_t step_lds = (size_t)(s.r + pl.dpad) * sizeof(double);
  bool done = false;
  const int *loop_error = nullptr;                           // set if the loop ran as resident launches (see k_gather)
  const void *fn = lp.fn;
  if (fn && one_slab_form) {
    SoloInit in;
    in.r_q = o->r_q; in.u = o->uniforms; in.scal = scal; in.tau_out = out->tau; in.seed = (unsigned long long)seed;
    in.rank_tol = s.rank_tol; in.tau_n = tau_n; in.beta = s.beta; in.bins = s.bins;
    int hcn = lp.hcn;
    void *args[] = {(void *)&a, (void *)&in, (void *)&hcn};
    const dim3 grid = lp.c.kind == kLoopWave ? dim3((P + kThreads / kWave - 1) / (kThreads / kWave)) : dim3(1, P);
    if (hipLaunchKernel(fn, grid, dim3(kThreads), args, lp.lds, st) != hipSuccess) return WILDCAT_EHIP;
    done = true;
  } else if (fn) {
    int *err_word = (int *)(ws + pl.off_sync);
    long long spin_limit = s.wait_limit > 0 ? s.wait_limit : 0;   // polls of about a microsecond each
    a.absent = s.wait_limit == -2 ? 2 : s.wait_limit < 0;
    int hcn = lp.hcn;
    // Ordinary launches, one per group of problems, back to back on the stream: a group was sized against the
    // device's capacity (choose_loop), so on an otherwise idle device every workgroup of a launch is resident at
    // once; if other work holds compute units, the late workgroups start when it ends and the resident ones poll
    // meanwhile (bounded).
    for (int g0 = 0; g0 < P; g0 += lp.c.group) {
      a.pr0 = g0;
      const int gp = P - g0 < lp.c.group ? P - g0 : lp.c.group;
      void *args[] = {(void *)&a, (void *)&err_word, (void *)&spin_limit, (void *)&hcn};
      if (hipLaunchKernel(fn, dim3(pl.nblk, gp), dim3(kThreads), args, lp.lds, st) != hipSuccess) return WILDCAT_EHIP;
    }
    a.pr0 = 0;
    loop_error = err_word;
    done = true;
  }
  if (!done) {
    for (int i = 0; i < s.r; ++i) {
      hipLaunchKernelGGL((k_step<T, KPT, H>), dim3(pl.nblk, P), dim3(kThreads), step_lds, st, a, i);
      LAUNCH_CHECK();
    }
  }
  if (o->ev_loop_end && hipEventRecord((hipEvent_t)o->ev_loop_end, st) != hipSuccess) return WILDCAT_EHIP;

  const int rtiles = (s.r + kGramRows - 1) / kGramRows;
  if (pl.gram_cols) {
    int tp = 64;
    while (tp < s.dv) tp <<= 1;
    const int sub = kThreads / tp;
    const dim3 grid((pl.nchunk + sub - 1) / sub, 1, P);
    const size_t run = (size_t)sub * pl.chunk_keys;            // <= 320 keys (n <= 256): at most 41 KB of LDS
    if (s.r <= 4)
      hipLaunchKernelGGL((k_gram_cols<T, 4, H>), grid, dim3(kThreads), (size_t)4 * run * sizeof(double), st, F, V, s.n,
                         pl.slab, s.r, s.dv, tp, (int)pl.chunk_keys, pl.nchunk, gpart);
    else if (s.r <= 8)
      hipLaunchKernelGGL((k_gram_cols<T, 8, H>), grid, dim3(kThreads), (size_t)8 * run * sizeof(double), st, F, V, s.n,
                         pl.slab, s.r, s.dv, tp, (int)pl.chunk_keys, pl.nchunk, gpart);
    else
      hipLaunchKernelGGL((k_gram_cols<T, 16, H>), grid, dim3(kThreads), (size_t)16 * run * sizeof(double), st, F, V, s.n,
                         pl.slab, s.r, s.dv, tp, (int)pl.chunk_keys, pl.nchunk, gpart);
  } else if (s.r <= 8 && s.dv % 8 == 0 && (s.dv / 8 & (s.dv / 8 - 1)) == 0 && s.dv <= 512 && pl.slab % 64 == 0 &&
             pl.chunk_keys % 64 == 0) {
    const int tpr = s.dv / 8;                                // threads per value row: a power of two, at most 64
    const dim3 grid(pl.nchunk, 1, P);
    if (s.r <= 4)
      hipLaunchKernelGGL((k_gram_small8<T, 4, H>), grid, dim3(kThreads), 0, st, F, V, s.n, pl.nblk, pl.slab, s.r, s.dv, tpr,
                         pl.chunk_keys, pl.nchunk, gpart);
    else
      hipLaunchKernelGGL((k_gram_small8<T, 8, H>), grid, dim3(kThreads), 0, st, F, V, s.n, pl.nblk, pl.slab, s.r, s.dv, tpr,
                         pl.chunk_keys, pl.nchunk, gpart);
  } else if (s.r <= 16) {
    int tpr = 1;
    while (tpr * 4 < s.dv) tpr <<= 1;                        // threads per value row (<= 64: dv <= kMaxWidth)
    const dim3 grid(pl.nchunk, 1, P);
    if (s.r <= 4)
      hipLaunchKernelGGL((k_gram_small<T, 4, H>), grid, dim3(kThreads), 0, st, F, V, s.n, pl.nblk, pl.slab, s.r, s.dv, tpr,
                         pl.chunk_keys, pl.nchunk, gpart);
    else if (s.r <= 8)
      hipLaunchKernelGGL((k_gram_small<T, 8, H>), grid, dim3(kThreads), 0, st, F, V, s.n, pl.nblk, pl.slab, s.r, s.dv, tpr,
                         pl.chunk_keys, pl.nchunk, gpart);
    else
      hipLaunchKernelGGL((k_gram_small<T, 16, H>), grid, dim3(kThreads), 0, st, F, V, s.n, pl.nblk, pl.slab, s.r, s.dv,
                         tpr, pl.chunk_keys, pl.nchunk, gpart);
  } else if (s.dv == 64 || s.dv == 128) {
    if (s.dv == 64)
      hipLaunchKernelGGL((k_gram_mfma<T, 4, H>), dim3(pl.nchunk, rtiles, P), dim3(kThreads), 0, st, F, V, s.n, pl.nblk,
                         pl.slab, s.r, pl.slabs_per_chunk, pl.nchunk, gpart);
    else
      hipLaunchKernelGGL((k_gram_mfma<T, 8, H>), dim3(pl.nchunk, rtiles, P), dim3(kThreads), 0, st, F, V, s.n, pl.nblk,
                         pl.slab, s.r, pl.slabs_per_chunk, pl.nchunk, gpart);
  } else if (s.dv == 256) {
    hipLaunchKernelGGL((k_gram_mfma<T, 16, H>), dim3(pl.nchunk, (s.r + 63) / 64, P), dim3(kThreads), 0, st, F, V, s.n,
                       pl.nblk, pl.slab, s.r, pl.slabs_per_chunk, pl.nchunk, gpart);
  } else if (s.dv <= 64) {
    hipLaunchKernelGGL((k_gram<T, 4, H>), dim3(pl.nchunk, rtiles, P), dim3(kThreads), 0, st, F, V, s.n, pl.nblk, pl.slab,
                       s.r, s.dv, pl.slabs_per_chunk, pl.nchunk, 1, gpart);
  } else {
    const int ncoltiles = (s.dv + 127) / 128;
    hipLaunchKernelGGL((k_gram<T, 8, H>), dim3(pl.nchunk * ncoltiles, rtiles, P), dim3(kThreads), 0, st, F, V, s.n,
                       pl.nblk, pl.slab, s.r, s.dv, pl.slabs_per_chunk, pl.nchunk, ncoltiles, gpart);
  }
  LAUNCH_CHECK();
  const int dv1 = s.dv + 1;
  if (s.r > kSolveSmall)
    hipLaunchKernelGGL(k_gram_reduce, dim3((s.r * dv1 + kThreads - 1) / kThreads, P), dim3(kThreads), 0, st, gpart, s.r,
                     dv1, pl.nchunk, Gt);
  LAUNCH_CHECK();
  if (s.r <= kSolveSmall) {
    const int64_t cols = (int64_t)P * dv1;
    hipLaunchKernelGGL(k_solve_small, dim3((unsigned)((cols + kThreads - 1) / kThreads)), dim3(kThreads), 0, st, L, gpart,
                       pl.nchunk, out->r_eff, P, s.r, s.dv, out->v_s, out->w);
  } else {
    const size_t solve_lds = ((size_t)kSolveCols * s.r + kPanel * (kPanel + 1) + kSolveCols * kPanel) * sizeof(double);
    if (solve_lds > 64 * 1024 &&
        hipFuncSetAttribute((const void *)k_solve, hipFuncAttributeMaxDynamicSharedMemorySize, (int)solve_lds) != hipSuccess)
      return WILDCAT_EHIP;
    hipLaunchKernelGGL(k_solve, dim3((dv1 + kSolveCols - 1) / kSolveCols, P), dim3(kSolveCols * 32), solve_lds, st, L, Gt,
                       out->r_eff, s.r, s.dv, out->v_s, out->w);
  }
  LAUNCH_CHECK();
  if (s.dtype == WILDCAT_BF16 && out->v_t && out->v_scale) {      // MFMA operand form of V_S for WtdAttn, per head
    const int rc = enqueue_pack_values(P / s.bins, s.r * s.bins, s.dv, out->v_s, out->v_t, out->v_scale, st);
    if (rc != WILDCAT_OK) return rc;
  }
  hipLaunchKernelGGL((k_gather<T>), dim3(s.r, P), dim3(64), 0, st, K, out->idx, s.n, s.d, s.r, s.bins,
                     (T *)out->k_s, loop_error, out->r_eff);
  LAUNCH_CHECK();
  if (out->W) {
    hipLaunchKernelGGL((k_debug_weights<H>), dim3((unsigned)((s.n + kThreads - 1) / kThreads), P), dim3(kThreads), 0, st, F, L,
                       out->r_eff, s.n, pl.nblk, pl.slab, s.r, out->W);
    LAUNCH_CHECK();
  }
  return WILDCAT_OK;
}

// Storage type T x keys per thread x history type H.
template <typename T, typename H>
int dispatch_kpt(const Shape &s, const Plan &pl, const void *K, const void *V, const wildcat_opts *o, uint64_t seed,
                 wildcat_coreset *out) {
  return pl.kpt == 2 ? run_compress<T, 2, H>(s, pl, (const T *)K, (const T *)V, o, seed, out)
                     : run_compress<T, 1, H>(s, pl, (const T *)K, (const T *)V, o, seed, out);
}
int dispatch_compress(const Shape &s, const Plan &pl, const void *K, const void *V, const wildcat_opts *o,
                      uint64_t seed, wildcat_coreset *out) {
  if (s.dtype == WILDCAT_BF16)
    return s.history_f32 ? dispatch_kpt<bf16_t, float>(s, pl, K, V, o, seed, out)
                         : dispatch_kpt<bf16_t, double>(s, pl, K, V, o, seed, out);
  return s.history_f32 ? dispatch_kpt<float, float>(s, pl, K, V, o, seed, out)
                       : dispatch_kpt<float, double>(s, pl, K, V, o, seed, out);
}
template <typename T, typename H>
LoopChoice loop_choice_kpt(const Shape &s, const Plan &pl) {
  return pl.kpt == 2 ? plan_loop<T, 2, H>(s, pl).c : plan_loop<T, 1, H>(s, pl).c;
}
LoopChoice dispatch_loop_choice(const Shape &s, const Plan &pl) {
  if (s.dtype == WILDCAT_BF16)
    return s.history_f32 ? loop_choice_kpt<bf16_t, float>(s, pl) : loop_choice_kpt<bf16_t, double>(s, pl);
  return s.history_f32 ? loop_choice_kpt<float, float>(s, pl) : loop_choice_kpt<float, double>(s, pl);
}

// Validation shared by the entry points that take a CompressKV shape; on success *s is the bin view.
int compress_shape(int64_t n, int32_t d, int32_t r, const wildcat_opts *opts, Shape *s) {
  Shape whole;
  const int rc = resolve_shape(n, 0, d, r, opts, &whole);
  if (rc != WILDCAT_OK) return rc;
  if (!bins_divide(whole)) return WILDCAT_EINVAL;
  *s = bin_view(whole);
  if (s->r > kMaxRank) return WILDCAT_EUNSUPPORTED;
  if (s->P > 65535 || (int64_t)s->P * s->r > INT32_MAX) return WILDCAT_EUNSUPPORTED;   // problems index grid.y / grid.z
  return WILDCAT_OK;
}

}  // namespace
}  // namespace wildcat

using namespace wildcat;

extern "C" int wildcat_compress_kv(const void *K, const void *V, int64_t n, int32_t d, int32_t r, uint64_t seed,
                                   const wildcat_opts *opts, wildcat_coreset *out) {
  if (!K || !V || !opts || !out) return WILDCAT_EINVAL;
  Shape s;
  const int rc = compress_shape(n, d, r, opts, &s);
  if (rc != WILDCAT_OK) return rc;
  if (!opts->r_q) return WILDCAT_EINVAL;
  if (!out->idx || !out->r_eff || !out->k_s || !out->v_s || !out->w || !out->v_min || !out->v_max || !out->tau)
    return WILDCAT_EINVAL;
  const Plan pl = make_plan(s);
  if (!opts->workspace || ((uintptr_t)opts->workspace & 255) || opts->workspace_bytes < pl.total)
    return WILDCAT_EWORKSPACE;
  return dispatch_compress(s, pl, K, V, opts, seed, out);
}

extern "C" int wildcat_rpnys_single_launch(int64_t n, int32_t d, int32_t r, const wildcat_opts *opts) {
  Shape s;
  const int rc = compress_shape(n, d, r, opts, &s);
  if (rc != WILDCAT_OK) return rc;
  return dispatch_loop_choice(s, make_plan(s)).kind != kLoopSteps ? 1 : 0;
}

extern "C" int wildcat_loop_plan(int64_t n, int32_t d, int32_t r, const wildcat_opts *opts, int32_t cus,
                                 int32_t occ_resident_keys, int32_t occ_streamed_keys, int32_t out[8]) {
  if (!out) return WILDCAT_EINVAL;
  Shape s;
  const int rc = compress_shape(n, d, r, opts, &s);
  if (rc != WILDCAT_OK) return rc;
  const Plan pl = make_plan(s);
  LoopChoice c;
  if (cus > 0) {
    if (occ_resident_keys < 0 || occ_streamed_keys < 0) return WILDCAT_EINVAL;
    const DeviceCaps caps = {cus, occ_resident_keys, occ_streamed_keys};
    c = choose_loop(s, pl, caps);
  } else {
    c = dispatch_loop_choice(s, pl);
  }
  out[0] = c.kind; out[1] = pl.kpt; out[2] = pl.nblk; out[3] = c.group; out[4] = c.kind == kLoopSteps ? 1 : c.launches;
  out[5] = c.keys_in_regs; out[6] = c.need; out[7] = 0;
  return WILDCAT_OK;
}
