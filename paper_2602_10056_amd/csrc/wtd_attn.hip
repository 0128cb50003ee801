// WtdAttn (Alg. 3) and the query radius R_Q of Alg. 4 for gfx950.
//
// WtdAttn is flash-attention shaped with a key length of only r: per query tile the coreset is streamed
// through LDS once, scores and the value product run on MFMA with fp32 accumulation, and a running
// maximum keeps exp() in range.  Any positive per-row factor cancels in Alg. 3's ratio and leaves the
// sign of the normaliser (A w) unchanged, so the max shift does not alter the "> 0" guard.
//
// Two kernels:
//   k_wtd_attn_mfma   bf16 storage.  Works on transposed tiles so that all softmax state of a query
//                     lives in one lane pair:  S^T = K_S Q^T  and  O^T = V_S^T P^T  with
//                     v_mfma_f32_32x32x16_bf16.  The normaliser sum_s P_s w_s is accumulated in fp32 on
//                     the vector ALU from the unrounded P (w may be negative and large).
//   k_wtd_attn_simple any storage type / width, fp32 arithmetic on the vector ALU (the fp32 path).
#include <cmath>

#include "common.h"

namespace wildcat {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
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
  if (threadIdx.x == 0) atomicMax(&acc[pr], (unsigned long long)__double_as_longlong(s));
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
                                                            unsigned long long *__restrict__ acc) {
  __shared__ double sm[kThreads / kWave];
  const int bh = blockIdx.y;
  const int b = bh / q_heads, hq = bh % q_heads;
  const int pr = b * (q_heads / group) + hq / group;
  const int rows_per_pass = kThreads / lpr;
  const int sub = threadIdx.x % lpr, rloc = threadIdx.x / lpr;
  const uint4 *base = reinterpret_cast<const uint4 *>(Q + (size_t)bh * m * d);
  double best = 0.0;
  for (int64_t row = (int64_t)blockIdx.x * rows_per_pass + rloc; row < m; row += (int64_t)gridDim.x * rows_per_pass) {
    double s = sumsq16(base[row * lpr + sub], T());
    for (int off = lpr / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, kWave);
    best = fmax(best, s);
  }
  best = block_reduce<double>(best, sm, MaxOp());
  if (threadIdx.x == 0) atomicMax(&acc[pr], (unsigned long long)__double_as_longlong(best));
}

__global__ void k_sqrt_inplace(double *x, int count) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < count) x[i] = sqrt(x[i]);
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
// bf16 MFMA kernel.  Workgroup = NW wavefronts, each owning 32 queries; key tiles of 64.
//
// v_mfma_f32_32x32x16_bf16 operand layout (lane l, g = l / 32):
//   A (32 x 16): row l % 32, k = 8 g .. 8 g + 7        B (16 x 32): column l % 32, k = 8 g .. 8 g + 7
//   D (32 x 32): column l % 32, register v holds row 8 (v / 4) + 4 g + (v % 4)
// S^T tile: rows = keys, columns = queries, so lane l holds 16 key scores of query l % 32 and lane l ^ 32
// the other 16.  Registers 8h .. 8h+7 of such a tile, converted to bf16, are used directly as the B
// operand of the value product; the A operand (V_S^T, rows = value columns) is read from LDS with the
// matching key order {16h + 4g + 0..3, 16h + 8 + 4g + 0..3}.
// --------------------------------------------------------------------------------------------
constexpr int kKT = 64;

template <int D, int DV, int NW>
__global__ __launch_bounds__(NW * kWave) void k_wtd_attn_mfma(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ Ks, const float *__restrict__ Vs,
    const float *__restrict__ w, const float *__restrict__ vmin, const float *__restrict__ vmax,
    const int32_t *__restrict__ r_eff, bf16_t *__restrict__ out, int64_t m, int r, int q_heads, int group,
    float scale_log2) {
  constexpr int KSTR = D + 8;       // bf16 elements per key row in LDS (16-byte pad against bank conflicts)
  constexpr int VSTR = kKT + 8;     // bf16 elements per value-column row in LDS
  constexpr int NT = NW * kWave;
  __shared__ __attribute__((aligned(16))) uint16_t lk[kKT * KSTR];
  __shared__ __attribute__((aligned(16))) uint16_t lv[DV * VSTR];
  __shared__ __attribute__((aligned(16))) float lw[kKT];

  const int t = threadIdx.x, wv = t / kWave, l = t % kWave, g = l / 32, c32 = l % 32;
  const int bh = blockIdx.y, b = bh / q_heads, hq = bh % q_heads;
  const int pr = b * (q_heads / group) + hq / group;
  const int64_t q0 = (int64_t)blockIdx.x * (NW * 32) + wv * 32;
  const int re = r_eff ? min(r_eff[pr], r) : r;

  // Q fragments (B operand of S^T = K Q^T): query c32, features 16 kb + 8 g .. + 7
  bf16x8 qf[D / 16];
  {
    const int64_t row = q0 + c32 < m ? q0 + c32 : m - 1;
    const uint4 *src = reinterpret_cast<const uint4 *>(Q + ((size_t)bh * m + row) * D + 8 * g);
#pragma unroll
    for (int kb = 0; kb < D / 16; ++kb) {
      const uint4 v = src[2 * kb];
      qf[kb] = *reinterpret_cast<const bf16x8 *>(&v);
    }
  }
  floatx16 acc[DV / 32];
#pragma unroll
  for (int i = 0; i < DV / 32; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
  float mrun = -INFINITY, den = 0.0f;

  const bf16_t *Kp = Ks + (size_t)pr * r * D;
  const float *Vp = Vs + (size_t)pr * r * DV;
  const float *wp = w + (size_t)pr * r;

  for (int k0 = 0; k0 < re; k0 += kKT) {
    __syncthreads();
    // ---- stage the key tile [64][D] (16-byte pieces) ------------------------------------------------
    for (int e = t; e < kKT * (D / 8); e += NT) {
      const int kk = e / (D / 8), seg = e % (D / 8);
      uint4 v = make_uint4(0, 0, 0, 0);
      if (k0 + kk < re) v = *reinterpret_cast<const uint4 *>(Kp + (size_t)(k0 + kk) * D + seg * 8);
      *reinterpret_cast<uint4 *>(&lk[kk * KSTR + seg * 8]) = v;
    }
    // ---- stage the value tile transposed, fp32 -> bf16: lv[col][key] -------------------------------------
    for (int e = t; e < kKT * (DV / 4); e += NT) {
      const int kk = e / (DV / 4), cs = e % (DV / 4);   // consecutive threads read one value row contiguously
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (k0 + kk < re) v = *reinterpret_cast<const float4 *>(Vp + (size_t)(k0 + kk) * DV + cs * 4);
      const floatx4 fv = {v.x, v.y, v.z, v.w};
      const bf16x4 bv = __builtin_convertvector(fv, bf16x4);
      const uint16_t *bits = reinterpret_cast<const uint16_t *>(&bv);
#pragma unroll
      for (int q = 0; q < 4; ++q) lv[(cs * 4 + q) * VSTR + kk] = bits[q];
    }
    if (t < kKT) lw[t] = k0 + t < re ? wp[k0 + t] : 0.0f;
    __syncthreads();

    // ---- S^T = K Q^T for the two 32-key halves ------------------------------------------------------------
    floatx16 st[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
      for (int v = 0; v < 16; ++v) st[mt][v] = 0.0f;
#pragma unroll
      for (int kb = 0; kb < D / 16; ++kb) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&lk[(32 * mt + c32) * KSTR + 16 * kb + 8 * g]);
        st[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kb], st[mt], 0, 0, 0);
      }
    }
    // ---- online softmax in the log2 domain ----------------------------------------------------------------
    float mx = -INFINITY;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = k0 + 32 * mt + 8 * (v / 4) + 4 * g + (v % 4);
        const float x = key < re ? st[mt][v] * scale_log2 : -INFINITY;
        st[mt][v] = x;
        mx = fmaxf(mx, x);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave));
    const float mnew = fmaxf(mrun, mx);
    const float alpha = __builtin_amdgcn_exp2f(mrun - mnew);
    mrun = mnew;
    float dl = 0.0f;
    bf16x8 pf[4];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      floatx16 p;
#pragma unroll
      for (int v = 0; v < 16; ++v) p[v] = __builtin_amdgcn_exp2f(st[mt][v] - mnew);
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 wv4 = *reinterpret_cast<const float4 *>(&lw[32 * mt + 8 * q + 4 * g]);
        dl = fmaf(p[4 * q + 0], wv4.x, dl);
        dl = fmaf(p[4 * q + 1], wv4.y, dl);
        dl = fmaf(p[4 * q + 2], wv4.z, dl);
        dl = fmaf(p[4 * q + 3], wv4.w, dl);
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const floatx8 ph = {p[8 * h + 0], p[8 * h + 1], p[8 * h + 2], p[8 * h + 3],
                            p[8 * h + 4], p[8 * h + 5], p[8 * h + 6], p[8 * h + 7]};
        pf[2 * mt + h] = __builtin_convertvector(ph, bf16x8);
      }
    }
    den = den * alpha + dl;
    if (alpha != 1.0f) {
#pragma unroll
      for (int i = 0; i < DV / 32; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] *= alpha;
    }
    // ---- O^T += V_S^T P^T ---------------------------------------------------------------------------------------
#pragma unroll
    for (int i = 0; i < DV / 32; ++i) {
#pragma unroll
      for (int kb = 0; kb < 4; ++kb) {
        const uint16_t *rowp = &lv[(32 * i + c32) * VSTR + 16 * kb + 4 * g];
        const uint2 lo = *reinterpret_cast<const uint2 *>(rowp);
        const uint2 hi = *reinterpret_cast<const uint2 *>(rowp + 8);
        const uint4 av = make_uint4(lo.x, lo.y, hi.x, hi.y);
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(&av), pf[kb], acc[i], 0, 0,
                                                         0);
      }
    }
  }
  // ---- epilogue: guard, divide, clip, store ------------------------------------------------------------------
  den += __shfl_xor(den, 32, kWave);
  const bool ok = den > 0.0f;
  const float inv = ok ? 1.0f / den : 0.0f;
  if (q0 + c32 < m) {
    bf16_t *orow = out + ((size_t)bh * m + q0 + c32) * DV;
#pragma unroll
    for (int i = 0; i < DV / 32; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = 32 * i + 8 * q + 4 * g;
        const float4 lo = *reinterpret_cast<const float4 *>(vmin + (size_t)pr * DV + col);
        const float4 hi = *reinterpret_cast<const float4 *>(vmax + (size_t)pr * DV + col);
        floatx4 o = {acc[i][4 * q + 0] * inv, acc[i][4 * q + 1] * inv, acc[i][4 * q + 2] * inv,
                     acc[i][4 * q + 3] * inv};
        if (!ok) o = {0.f, 0.f, 0.f, 0.f};
        o[0] = fminf(fmaxf(o[0], lo.x), hi.x);
        o[1] = fminf(fmaxf(o[1], lo.y), hi.y);
        o[2] = fminf(fmaxf(o[2], lo.z), hi.z);
        o[3] = fminf(fmaxf(o[3], lo.w), hi.w);
        const bf16x4 ob = __builtin_convertvector(o, bf16x4);
        *reinterpret_cast<uint2 *>(orow + col) = *reinterpret_cast<const uint2 *>(&ob);
      }
  }
}


// --------------------------------------------------------------------------------------------
// Pipelined bf16 MFMA kernel (needs the transposed bf16 values v_t of the coreset).
// Workgroup = 8 wavefronts (two per SIMD, so one wave's exp/convert work overlaps the other's MFMAs), each
// owning 32 queries.  Key tiles of 64 are double-buffered in LDS: the loads of tile t+1 are issued before the
// math of tile t and stored after it, with one barrier per tile.  Same operand layouts as above.
//
// The running maximum is only a reference point for exp(): any reference within 2^8 of the true row maximum
// keeps every exponential in range, and a change of reference multiplies numerator and normaliser of a row
// alike.  So the accumulators are rescaled only when a row's maximum has grown by more than 8 (log2 units)
// since its reference was set -- rare after the first tile -- instead of on every tile.
// --------------------------------------------------------------------------------------------
constexpr float kRescaleSlack = 8.0f;

template <int D, int DV>
__global__ __launch_bounds__(512, 1) void k_wtd_attn_mfma2(
    const bf16_t *__restrict__ Q, const bf16_t *__restrict__ Ks, const bf16_t *__restrict__ Vt,
    const float *__restrict__ w, const float *__restrict__ vmin, const float *__restrict__ vmax,
    const int32_t *__restrict__ r_eff, bf16_t *__restrict__ out, int64_t m, int r, int r64, int q_heads, int group,
    float scale_log2) {
  constexpr int KSTR = D + 8;        // bf16 per key row in LDS
  constexpr int VSTR = kKT + 8;      // bf16 per value-column row in LDS
  constexpr int NT = 512;
  constexpr int KPIECES = (kKT * D / 8 + NT - 1) / NT;     // 16-byte pieces of the key tile per thread
  constexpr int VPIECES = (DV * kKT / 8 + NT - 1) / NT;    // 16-byte pieces of the value tile per thread
  __shared__ __attribute__((aligned(16))) uint16_t lk[2][kKT * KSTR];
  __shared__ __attribute__((aligned(16))) uint16_t lv[2][DV * VSTR];
  __shared__ __attribute__((aligned(16))) float lw[2][kKT];

  const int t = threadIdx.x, wv = t / kWave, l = t % kWave, g = l / 32, c32 = l % 32;
  const int bh = blockIdx.y, b = bh / q_heads, hq = bh % q_heads;
  const int pr = b * (q_heads / group) + hq / group;
  const int64_t q0 = (int64_t)blockIdx.x * 256 + wv * 32;
  const int re = r_eff ? min(r_eff[pr], r) : r;
  const bf16_t *Kp = Ks + (size_t)pr * r * D;
  const bf16_t *Vp = Vt + (size_t)pr * DV * r64;
  const float *wp = w + (size_t)pr * r;

  uint4 kst[KPIECES], vst[VPIECES];
  float wst = 0.0f;
  auto fetch = [&](int k0) {
#pragma unroll
    for (int e = 0; e < KPIECES; ++e) {
      const int idx = t + e * NT, kk = idx / (D / 8), seg = idx % (D / 8);
      kst[e] = (idx < kKT * D / 8 && k0 + kk < re)
                   ? *reinterpret_cast<const uint4 *>(Kp + (size_t)(k0 + kk) * D + seg * 8)
                   : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int e = 0; e < VPIECES; ++e) {
      const int idx = t + e * NT, col = idx / (kKT / 8), seg = idx % (kKT / 8);
      vst[e] = idx < DV * kKT / 8 ? *reinterpret_cast<const uint4 *>(Vp + (size_t)col * r64 + k0 + seg * 8)
                                  : make_uint4(0, 0, 0, 0);
    }
    if (t < kKT) wst = k0 + t < re ? wp[k0 + t] : 0.0f;
  };
  auto stash = [&](int buf) {
#pragma unroll
    for (int e = 0; e < KPIECES; ++e) {
      const int idx = t + e * NT, kk = idx / (D / 8), seg = idx % (D / 8);
      if (idx < kKT * D / 8) *reinterpret_cast<uint4 *>(&lk[buf][kk * KSTR + seg * 8]) = kst[e];
    }
#pragma unroll
    for (int e = 0; e < VPIECES; ++e) {
      const int idx = t + e * NT, col = idx / (kKT / 8), seg = idx % (kKT / 8);
      if (idx < DV * kKT / 8) *reinterpret_cast<uint4 *>(&lv[buf][col * VSTR + seg * 8]) = vst[e];
    }
    if (t < kKT) lw[buf][t] = wst;
  };

  fetch(0);
  // Q fragments: B operand of S^T = K Q^T: query c32, features 16 kb + 8 g .. + 7
  bf16x8 qf[D / 16];
  {
    const int64_t row = q0 + c32 < m ? q0 + c32 : m - 1;
    const uint4 *src = reinterpret_cast<const uint4 *>(Q + ((size_t)bh * m + row) * D + 8 * g);
#pragma unroll
    for (int kb = 0; kb < D / 16; ++kb) {
      const uint4 v = src[2 * kb];
      qf[kb] = *reinterpret_cast<const bf16x8 *>(&v);
    }
  }
  floatx16 acc[DV / 32];
#pragma unroll
  for (int i = 0; i < DV / 32; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
  float mref = -INFINITY, den = 0.0f;      // reference exponent (log2 domain) and normaliser of query c32
  stash(0);
  __syncthreads();

  int buf = 0;
  for (int k0 = 0; k0 < re; k0 += kKT, buf ^= 1) {
    const bool more = k0 + kKT < re;
    if (more) fetch(k0 + kKT);
    // ---- S^T = K Q^T for the two 32-key halves -----------------------------------------------------------
    floatx16 st[2];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) st[mt][v] = 0.0f;
#pragma unroll
    for (int kb = 0; kb < D / 16; ++kb) {
#pragma unroll
      for (int mt = 0; mt < 2; ++mt) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&lk[buf][(32 * mt + c32) * KSTR + 16 * kb + 8 * g]);
        st[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kb], st[mt], 0, 0, 0);
      }
    }
    if (k0 + kKT > re) {                                     // ragged last tile: mask the missing keys
#pragma unroll
      for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (k0 + 32 * mt + 8 * (v / 4) + 4 * g + (v % 4) >= re) st[mt][v] = -INFINITY;
    }
    // ---- row maximum of the raw scores; move the reference only if it is more than the slack behind ------------
    float mx = st[0][0];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, st[mt][v]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, kWave)) * scale_log2;
    const bool jump = mx > mref + kRescaleSlack;
    if (__builtin_amdgcn_ballot_w64(jump) != 0) {
      const float alpha = jump ? __builtin_amdgcn_exp2f(mref - mx) : 1.0f;
      mref = jump ? mx : mref;
      den *= alpha;
#pragma unroll
      for (int i = 0; i < DV / 32; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] *= alpha;
    }
    // ---- P = exp2(S c - mref), normaliser, bf16 operand ---------------------------------------------------------
    const float nm = -mref;
    float dl = 0.0f;
    bf16x8 pf[4];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
      floatx16 p;
#pragma unroll
      for (int v = 0; v < 16; ++v) p[v] = __builtin_amdgcn_exp2f(fmaf(st[mt][v], scale_log2, nm));
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float4 wv4 = *reinterpret_cast<const float4 *>(&lw[buf][32 * mt + 8 * q + 4 * g]);
        dl = fmaf(p[4 * q + 0], wv4.x, dl);
        dl = fmaf(p[4 * q + 1], wv4.y, dl);
        dl = fmaf(p[4 * q + 2], wv4.z, dl);
        dl = fmaf(p[4 * q + 3], wv4.w, dl);
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const floatx8 ph = {p[8 * h + 0], p[8 * h + 1], p[8 * h + 2], p[8 * h + 3],
                            p[8 * h + 4], p[8 * h + 5], p[8 * h + 6], p[8 * h + 7]};
        pf[2 * mt + h] = __builtin_convertvector(ph, bf16x8);
      }
    }
    den += dl;
    // ---- O^T += V_S^T P^T ------------------------------------------------------------------------------------
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
#pragma unroll
      for (int i = 0; i < DV / 32; ++i) {
        const uint16_t *rowp = &lv[buf][(32 * i + c32) * VSTR + 16 * kb + 4 * g];
        const uint2 lo = *reinterpret_cast<const uint2 *>(rowp);
        const uint2 hi = *reinterpret_cast<const uint2 *>(rowp + 8);
        const uint4 av = make_uint4(lo.x, lo.y, hi.x, hi.y);
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(&av), pf[kb], acc[i], 0, 0,
                                                         0);
      }
    }
    if (more) stash(buf ^ 1);
    __syncthreads();
  }
  // ---- epilogue: guard, divide, clip, store -------------------------------------------------------------------
  den += __shfl_xor(den, 32, kWave);
  const bool ok = den > 0.0f;
  const float inv = ok ? 1.0f / den : 0.0f;
  if (q0 + c32 < m) {
    bf16_t *orow = out + ((size_t)bh * m + q0 + c32) * DV;
#pragma unroll
    for (int i = 0; i < DV / 32; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = 32 * i + 8 * q + 4 * g;
        const float4 lo = *reinterpret_cast<const float4 *>(vmin + (size_t)pr * DV + col);
        const float4 hi = *reinterpret_cast<const float4 *>(vmax + (size_t)pr * DV + col);
        floatx4 o = {acc[i][4 * q + 0] * inv, acc[i][4 * q + 1] * inv, acc[i][4 * q + 2] * inv,
                     acc[i][4 * q + 3] * inv};
        if (!ok) o = {0.f, 0.f, 0.f, 0.f};
        o[0] = fminf(fmaxf(o[0], lo.x), hi.x);
        o[1] = fminf(fmaxf(o[1], lo.y), hi.y);
        o[2] = fminf(fmaxf(o[2], lo.z), hi.z);
        o[3] = fminf(fmaxf(o[3], lo.w), hi.w);
        const bf16x4 ob = __builtin_convertvector(o, bf16x4);
        *reinterpret_cast<uint2 *>(orow + col) = *reinterpret_cast<const uint2 *>(&ob);
      }
  }
}

// v_t[pr][c][j] = bf16(v_s[pr][j][c]) for j < r, zero for r <= j < r64.  grid (ceil(r64*dv/256), P).
__global__ __launch_bounds__(kThreads) void k_pack_values(const float *__restrict__ v_s, int r, int r64, int dv,
                                                          bf16_t *__restrict__ v_t) {
  const int pr = blockIdx.y;
  const int gid = blockIdx.x * kThreads + threadIdx.x;
  if (gid >= r64 * dv) return;
  const int c = gid / r64, j = gid % r64;
  from_float(j < r ? v_s[((size_t)pr * r + j) * dv + c] : 0.0f, &v_t[((size_t)pr * dv + c) * r64 + j]);
}

template <int D, int DV>
int launch_mfma2(const Shape &s, const void *Q, const wildcat_coreset *cs, void *out) {
  const int r64 = (s.r + 63) / 64 * 64;
  const dim3 grid((unsigned)((s.m + 255) / 256), s.batch * s.q_heads);
  hipLaunchKernelGGL((k_wtd_attn_mfma2<D, DV>), grid, dim3(512), 0, s.stream, (const bf16_t *)Q,
                     (const bf16_t *)cs->k_s, (const bf16_t *)cs->v_t, cs->w, cs->v_min, cs->v_max, cs->r_eff,
                     (bf16_t *)out, s.m, s.r, r64, s.q_heads, s.group, (float)(s.beta * (double)kLog2e));
  return hipGetLastError() == hipSuccess ? WILDCAT_OK : WILDCAT_EHIP;
}

template <int D, int DV>
int launch_mfma(const Shape &s, const void *Q, const wildcat_coreset *cs, void *out) {
  constexpr int NW = 4;
  const dim3 grid((unsigned)((s.m + NW * 32 - 1) / (NW * 32)), s.batch * s.q_heads);
  hipLaunchKernelGGL((k_wtd_attn_mfma<D, DV, NW>), grid, dim3(NW * kWave), 0, s.stream, (const bf16_t *)Q,
                     (const bf16_t *)cs->k_s, cs->v_s, cs->w, cs->v_min, cs->v_max, cs->r_eff, (bf16_t *)out, s.m, s.r,
                     s.q_heads, s.group, (float)(s.beta * (double)kLog2e));
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
}  // namespace wildcat

using namespace wildcat;

extern "C" int wildcat_query_radius(const void *Q, int64_t m, int32_t d, const wildcat_opts *opts, double *r_q_out) {
  if (!Q || !r_q_out || m < 1) return WILDCAT_EINVAL;
  Shape s;
  int rc = resolve_shape(m, m, d, 1, opts, &s);
  if (rc != WILDCAT_OK) return rc;
  hipLaunchKernelGGL(k_zero_u64, dim3((s.P + 255) / 256), dim3(256), 0, s.stream, (unsigned long long *)r_q_out, s.P);
  if (hipGetLastError() != hipSuccess) return WILDCAT_EHIP;
  const int es = s.dtype == WILDCAT_BF16 ? 2 : 4;
  const int pieces = (d * es) % 16 == 0 ? d * es / 16 : 0;
  if (pieces >= 1 && pieces <= kWave && (pieces & (pieces - 1)) == 0) {
    const int rows_per_pass = kThreads / pieces;
    int64_t blocks = (m + rows_per_pass - 1) / rows_per_pass;
    const int64_t cap = (4096 + s.batch * s.q_heads - 1) / (s.batch * s.q_heads);
    if (blocks > cap) blocks = cap;
    const dim3 grid((unsigned)blocks, s.batch * s.q_heads);
    if (s.dtype == WILDCAT_BF16)
      hipLaunchKernelGGL((k_qnorm_max_vec<bf16_t>), grid, dim3(kThreads), 0, s.stream, (const bf16_t *)Q, m, d, pieces,
                         s.q_heads, s.group, (unsigned long long *)r_q_out);
    else
      hipLaunchKernelGGL((k_qnorm_max_vec<float>), grid, dim3(kThreads), 0, s.stream, (const float *)Q, m, d, pieces,
                         s.q_heads, s.group, (unsigned long long *)r_q_out);
  } else {
    const dim3 grid((unsigned)((m + kThreads - 1) / kThreads), s.batch * s.q_heads);
    if (s.dtype == WILDCAT_BF16)
      hipLaunchKernelGGL((k_qnorm_max<bf16_t>), grid, dim3(kThreads), 0, s.stream, (const bf16_t *)Q, m, d, s.q_heads,
                         s.group, (unsigned long long *)r_q_out);
    else
      hipLaunchKernelGGL((k_qnorm_max<float>), grid, dim3(kThreads), 0, s.stream, (const float *)Q, m, d, s.q_heads,
                         s.group, (unsigned long long *)r_q_out);
  }
  if (hipGetLastError() != hipSuccess) return WILDCAT_EHIP;
  hipLaunchKernelGGL(k_sqrt_inplace, dim3((s.P + 255) / 256), dim3(256), 0, s.stream, r_q_out, s.P);
  return hipGetLastError() == hipSuccess ? WILDCAT_OK : WILDCAT_EHIP;
}

extern "C" int wildcat_wtd_attn(const void *Q, const wildcat_coreset *cs, void *out, int64_t m, int32_t d, int32_t r,
                                const wildcat_opts *opts) {
  if (!Q || !cs || !out || m < 1 || r < 1) return WILDCAT_EINVAL;
  if (!cs->k_s || !cs->v_s || !cs->w || !cs->v_min || !cs->v_max) return WILDCAT_EINVAL;
  Shape s;
  int rc = resolve_shape(r, m, d, r, opts, &s);
  if (rc != WILDCAT_OK) return rc;
  if (s.dtype == WILDCAT_BF16) {
    if (cs->v_t) {
      if (s.d == 64 && s.dv == 64) return launch_mfma2<64, 64>(s, Q, cs, out);
      if (s.d == 128 && s.dv == 128) return launch_mfma2<128, 128>(s, Q, cs, out);
    }
    if (s.d == 64 && s.dv == 64) return launch_mfma<64, 64>(s, Q, cs, out);
    if (s.d == 128 && s.dv == 128) return launch_mfma<128, 128>(s, Q, cs, out);
    if (s.d == 64 && s.dv == 128) return launch_mfma<64, 128>(s, Q, cs, out);
    if (s.d == 64 && s.dv == 256) return launch_mfma<64, 256>(s, Q, cs, out);
    return launch_simple<bf16_t>(s, Q, cs, out);
  }
  return launch_simple<float>(s, Q, cs, out);
}

extern "C" int wildcat_pack_values(const wildcat_coreset *cs, int32_t r, int32_t dv, const wildcat_opts *opts) {
  if (!cs || !cs->v_s || !cs->v_t || r < 1 || dv < 1) return WILDCAT_EINVAL;
  Shape s;
  int rc = resolve_shape(r, 0, dv, r, opts, &s);
  if (rc != WILDCAT_OK) return rc;
  if (s.dtype != WILDCAT_BF16) return WILDCAT_EINVAL;
  const int r64 = (r + 63) / 64 * 64;
  hipLaunchKernelGGL(k_pack_values, dim3((r64 * dv + kThreads - 1) / kThreads, s.P), dim3(kThreads), 0, s.stream,
                     cs->v_s, r, r64, dv, (bf16_t *)cs->v_t);
  return hipGetLastError() == hipSuccess ? WILDCAT_OK : WILDCAT_EHIP;
}
