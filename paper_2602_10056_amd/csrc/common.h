// Internal helpers shared by the libwildcat translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "wildcat.h"

namespace wildcat {

constexpr int kThreads = 256;       // workgroup size of every streaming kernel (4 wavefronts of 64)
constexpr int kWave = 64;
constexpr int kMaxWidth = 256;      // largest key / value width d, dv
constexpr int kMaxRank = 2048;      // largest coreset size r (the core solve keeps 8 columns of r doubles in LDS)
constexpr int kChunk = 4;           // keys are re-packed as [d/4][n][4] for coalesced per-key access

// Pivot records (resident loop): the record of step i holds i + dpad + 4 doubles -- g_0 .. g_{i-1}, k_s - kbar,
// p_s, <kbar, k_s - kbar>, two spare -- and the records of a problem lie one after the other.  A word that has not
// been written yet holds the all-ones pattern (k_init_p fills them; no arithmetic produces that NaN, and widening a
// narrower NaN leaves low zero bits), so every word says for itself whether it has arrived.
__host__ __device__ inline size_t mail_offset(int i, int dpad) { return (size_t)i * (i - 1) / 2 + (size_t)i * (dpad + 4); }
__host__ __device__ inline size_t mail_words(int r, int dpad) { return mail_offset(r, dpad); }
constexpr long long kMailEmpty = -1;


// ---- resolved options -------------------------------------------------------------------------
struct Shape {
  int batch, q_heads, kv_heads, group, P;
  int64_t n, m;
  int d, dv, r, dtype;
  int bins;          // B of Alg. 2 (>= 1)
  int tau_full_n;    // temperature from the full length n instead of the bin length n / B
  int history_f32;   // history rows of the selection loop in fp32 (fast mode) instead of fp64
  int loop_driver;   // wildcat_loop: how the selection loop is launched
  long long wait_limit;  // polls before a wait inside the resident loop gives up (> 0), or the test hook (< 0)
  double beta, rank_tol;
  hipStream_t stream;
};

// The bin loop of Alg. 2 as a batch: the same shape with every bin as a problem of its own
// (P * B problems of n / B keys and r / B pivots; contiguous bins are a reshape of K and V).  `bins` is kept.
// Bins are equal, contiguous blocks of rows with equal shares of the rank: B must divide n and r.
inline bool bins_divide(const Shape &s) { return s.n % s.bins == 0 && s.r % s.bins == 0; }

inline Shape bin_view(const Shape &s) {
  Shape v = s;
  v.P = s.P * s.bins;
  v.n = s.n / s.bins;
  v.r = s.r / s.bins;
  return v;
}

// Fills `s` from the raw arguments with the defaults of wildcat_opts; returns a wildcat_status.
int resolve_shape(int64_t n, int64_t m_arg, int32_t d, int32_t r, const wildcat_opts *o, Shape *s);

// ---- workspace plan of CompressKV --------------------------------------------------------------
struct Plan {
  int kpt;          // keys per thread in the step kernel (1 or 2)
  int slab;         // keys per workgroup = kThreads * kpt
  int nblk;         // slabs per problem
  int64_t npad;     // nblk * slab
  int dpad;         // d rounded up to a multiple of kChunk
  int nb0;          // row blocks of the column-statistics pass
  int nchunk;       // n-chunks of the Gram pass
  int slabs_per_chunk;
  int64_t chunk_keys;  // keys per chunk: slabs_per_chunk * slab, or a piece of the bin (gram_cols)
  bool gram_cols;      // small bins of small rank: the Gram pass runs as k_gram_cols
  size_t off_kbar, off_kp, off_d0, off_p, off_bsum, off_scal, off_F, off_L, off_gpart, off_g,
      off_mpart, off_vminpart, off_vmaxpart, off_u, off_sync, off_mail;
  bool persistent;  // the selection loop may run as resident launches (see choose_loop); false: one launch per step
  size_t total;
};
Plan make_plan(const Shape &s);

// ---- how the selection loop (Alg. 1) of a shape is launched ------------------------------------------------
enum LoopKind {
  kLoopSteps = 0,     // one launch per step: the kernel boundary synchronises the slabs of a problem
  kLoopResident = 1,  // all steps in one launch per group of problems; the slabs of a problem poll each other
  kLoopSolo = 2,      // problems of one slab: one workgroup alone with its problem, one launch, nothing polled
  kLoopWave = 3       // tiny problems: one wavefront per problem, one launch
};
struct DeviceCaps {
  int cus;         // compute units
  int occ_regs;    // workgroups of the loop kernel a compute unit holds with the keys kept in registers (0: none)
  int occ_stream;  // ... with the keys streamed from memory every step
};
struct LoopChoice {
  int kind;          // LoopKind
  int keys_in_regs;  // the keys stay in registers for the whole loop
  int group;         // problems per launch
  int launches;      // launches for all problems (kLoopSteps: per step)
  int need;          // workgroups a compute unit must hold during a launch
};
// Pure host logic (no device is touched): the launch form of the loop for shape `s` (the bin view) on a device with
// the given capacities.
LoopChoice choose_loop(const Shape &s, const Plan &pl, const DeviceCaps &caps, bool allow_wave = true);
// Whether a loop kernel that keeps the packed keys in registers exists for this storage type, keys per thread and
// padded width; whether the wavefront-per-problem loop covers this shape.
bool keys_fit_registers(int dtype, int kpt, int dpad);
bool wave_loop_covers(const Shape &s, int dpad);

// Number of compute units of the current device.
int compute_units();

// Writes the packed half-precision values v_t and their scale v_scale (see wildcat_coreset) from v_s [P, r, dv].
int enqueue_pack_values(int P, int r, int dv, const float *v_s, void *v_t, float *v_scale, hipStream_t stream);

// ---- storage types ---------------------------------------------------------------------------
struct bf16_t { uint16_t bits; };

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return __uint_as_float(((uint32_t)x.bits) << 16); }

__device__ __forceinline__ void from_float(float v, float *dst) { *dst = v; }
__device__ __forceinline__ void from_float(float v, bf16_t *dst) {   // round to nearest even
  uint32_t u = __float_as_uint(v);
  if ((u & 0x7fffffffu) > 0x7f800000u) { dst->bits = (uint16_t)((u >> 16) | 0x40); return; }
  u += 0x7fffu + ((u >> 16) & 1u);
  dst->bits = (uint16_t)(u >> 16);
}

// ---- deterministic workgroup reductions / scans over kThreads threads ------------------------------------
// All take one value per thread and combine in a fixed order, so results do not depend on timing.

// The cross-lane steps are data-parallel-primitive moves (shifts inside rows of 16 lanes, then lane 15 of a row
// broadcast to the next row and lane 31 to the upper half): they stay inside the vector unit, where a shuffle goes
// through the LDS crossbar and costs a round trip per step -- six to twelve of them per scan or reduction, several
// scans and reductions per step of the selection loop.
//   dpp_move<CTRL, ROWS>(fill, x): lane l receives x of the lane CTRL names, or `fill` where that lane does not exist
//   or l's row is not in the row mask ROWS.
constexpr int kDppRowShr = 0x110, kDppWaveShr1 = 0x138, kDppRowBcast15 = 0x142, kDppRowBcast31 = 0x143;
template <int CTRL, int ROWS = 0xf>
__device__ __forceinline__ int dpp_move(int fill, int x) {
  return __builtin_amdgcn_update_dpp(fill, x, CTRL, ROWS, 0xf, false);
}
template <int CTRL, int ROWS = 0xf>
__device__ __forceinline__ double dpp_move(double fill, double x) {
  const int lo = __builtin_amdgcn_update_dpp(__double2loint(fill), __double2loint(x), CTRL, ROWS, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(__double2hiint(fill), __double2hiint(x), CTRL, ROWS, 0xf, false);
  return __hiloint2double(hi, lo);
}
// Inclusive scan of a wavefront under an associative op with identity `id` (lane l: op over lanes 0 .. l).
template <typename T, typename Op>
__device__ __forceinline__ T wave_incl_scan_op(T v, T id, Op op) {
  v = op(v, dpp_move<kDppRowShr + 1>(id, v));
  v = op(v, dpp_move<kDppRowShr + 2>(id, v));
  v = op(v, dpp_move<kDppRowShr + 4>(id, v));
  v = op(v, dpp_move<kDppRowShr + 8>(id, v));
  v = op(v, dpp_move<kDppRowBcast15, 0xa>(id, v));           // rows 1 and 3 take the total of the row below
  v = op(v, dpp_move<kDppRowBcast31, 0xc>(id, v));           // rows 2 and 3 take the total of the lower half
  return v;
}
struct AddOp { template <typename T> __device__ T operator()(T a, T b) const { return a + b; } };
__device__ __forceinline__ double wave_incl_scan(double v) { return wave_incl_scan_op(v, 0.0, AddOp()); }

// Inclusive scan across the workgroup; *total receives the sum of all values.  `sm` is >= 4 doubles of LDS.
__device__ __forceinline__ double block_incl_scan(double v, double *sm, double *total) {
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
  double inc = wave_incl_scan(v);
  __syncthreads();                       // protect sm from a previous use
  if (lane == kWave - 1) sm[wv] = inc;
  __syncthreads();
  double base = 0.0, tot = 0.0;
#pragma unroll
  for (int k = 0; k < kThreads / kWave; ++k) {
    double x = sm[k];
    if (k < wv) base += x;
    tot += x;
  }
  *total = tot;
  return base + inc;
}

__device__ __forceinline__ double block_sum(double v, double *sm) {
  double tot;
  block_incl_scan(v, sm, &tot);
  return tot;
}

// (min or max: the value itself serves as the fill of the scan -- combining a value with itself changes nothing)
template <typename T, typename Op>
__device__ __forceinline__ T block_reduce(T v, T *sm, Op op) {
  const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
  v = op(v, dpp_move<kDppRowShr + 1>(v, v));
  v = op(v, dpp_move<kDppRowShr + 2>(v, v));
  v = op(v, dpp_move<kDppRowShr + 4>(v, v));
  v = op(v, dpp_move<kDppRowShr + 8>(v, v));
  v = op(v, dpp_move<kDppRowBcast15, 0xa>(v, v));
  v = op(v, dpp_move<kDppRowBcast31, 0xc>(v, v));            // lane 63 now holds the wavefront's result
  __syncthreads();
  if (lane == kWave - 1) sm[wv] = v;
  __syncthreads();
  T out = sm[0];
#pragma unroll
  for (int k = 1; k < kThreads / kWave; ++k) out = op(out, sm[k]);
  return out;
}

struct MinOp { template <typename T> __device__ T operator()(T a, T b) const { return a < b ? a : b; } };
struct MaxOp { template <typename T> __device__ T operator()(T a, T b) const { return a > b ? a : b; } };

// ---- host-side launch check ------------------------------------------------------------------
inline int hip_ok(hipError_t e) { return e == hipSuccess ? WILDCAT_OK : WILDCAT_EHIP; }

}  // namespace wildcat
