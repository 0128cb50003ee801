// Host-side pieces of the C ABI that launch nothing: option resolution, the workspace plan,
// the documented uniform stream and error strings.
#include <cmath>
#include <cstring>

#include "common.h"

namespace wildcat {

int resolve_shape(int64_t n, int64_t m_arg, int32_t d, int32_t r, const wildcat_opts *o, Shape *s) {
  wildcat_opts z = {};
  if (!o) o = &z;
  s->batch = o->batch > 0 ? o->batch : 1;
  s->kv_heads = o->kv_heads > 0 ? o->kv_heads : 1;
  s->q_heads = o->q_heads > 0 ? o->q_heads : s->kv_heads;
  if (o->batch < 0 || o->kv_heads < 0 || o->q_heads < 0) return WILDCAT_EINVAL;
  if (s->q_heads % s->kv_heads) return WILDCAT_EINVAL;
  s->group = s->q_heads / s->kv_heads;
  if ((int64_t)s->batch * s->kv_heads > (1 << 20)) return WILDCAT_EINVAL;
  s->P = s->batch * s->kv_heads;
  if (n < 1 || n > (int64_t)1 << 30 || d < 1 || r < 1 || r > n) return WILDCAT_EINVAL;
  if (o->dv < 0 || o->m < 0 || m_arg < 0) return WILDCAT_EINVAL;
  s->n = n;
  s->m = m_arg > 0 ? m_arg : (o->m > 0 ? o->m : n);
  if (s->m > (int64_t)1 << 30) return WILDCAT_EINVAL;
  s->d = d;
  s->dv = o->dv > 0 ? o->dv : d;
  s->r = r;
  if (o->dtype != WILDCAT_F32 && o->dtype != WILDCAT_BF16) return WILDCAT_EINVAL;
  s->dtype = o->dtype;
  if (!(o->beta >= 0.0) || !std::isfinite(o->beta)) return WILDCAT_EINVAL;
  s->beta = o->beta > 0.0 ? o->beta : 1.0 / std::sqrt((double)d);
  if (!std::isfinite(o->rank_tol) || o->rank_tol >= 1.0) return WILDCAT_EINVAL;
  s->rank_tol = o->rank_tol == 0.0 ? 1e-10 : (o->rank_tol < 0.0 ? 0.0 : o->rank_tol);
  if (o->bins < 0 || o->tau_length < 0 || o->tau_length > 1) return WILDCAT_EINVAL;
  s->bins = o->bins > 1 ? o->bins : 1;
  s->tau_full_n = o->tau_length;
  if (o->history != WILDCAT_HISTORY_F64 && o->history != WILDCAT_HISTORY_F32) return WILDCAT_EINVAL;
  s->history_f32 = o->history == WILDCAT_HISTORY_F32;
  if (o->loop_driver < WILDCAT_LOOP_AUTO || o->loop_driver > WILDCAT_LOOP_WAVE) return WILDCAT_EINVAL;
  s->loop_driver = o->loop_driver;
  s->wait_limit = o->wait_limit == 0 ? 2000000ll : (long long)o->wait_limit;
  if ((int64_t)s->P * s->bins > (1 << 20)) return WILDCAT_EINVAL;
  if (d > kMaxWidth || s->dv > kMaxWidth) return WILDCAT_EUNSUPPORTED;
  s->stream = (hipStream_t)o->stream;
  return WILDCAT_OK;
}

int compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  return (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) ? n : 256;
}

bool keys_fit_registers(int dtype, int kpt, int dpad) {
  // 32-bit registers per chunk of four features: bf16 pairs stay packed; at most 128 registers for the keys
  const int nc = dpad / kChunk, regs_per_chunk = kpt * (dtype == WILDCAT_BF16 ? 2 : 4);
  return (nc == 32 || nc == 16) && nc * regs_per_chunk <= 128;
}

bool wave_loop_covers(const Shape &s, int dpad) {
  return s.r <= 16 && ((dpad == 64 && s.n <= 128) || (dpad == 128 && s.n <= 64));
}

LoopChoice choose_loop(const Shape &s, const Plan &pl, const DeviceCaps &caps, bool allow_wave) {
  const LoopChoice steps = {kLoopSteps, 0, s.P, 1, 0};
  if (!pl.persistent || s.loop_driver == WILDCAT_LOOP_STEPS || caps.cus < 1) return steps;
  const int occ_regs = keys_fit_registers(s.dtype, pl.kpt, pl.dpad) ? caps.occ_regs : 0;
  if (pl.nblk == 1) {
    // One slab per problem: no workgroup waits for another, so any number of them may be queued in one launch.
    // One wave per problem pays once the workgroup-per-problem form would need several rounds of workgroups: a
    // wave alone takes about 6 us per step against 4 us for a workgroup, but sixteen times as many are in flight.
    if (allow_wave && wave_loop_covers(s, pl.dpad) && (s.P > 2 * caps.cus || s.loop_driver == WILDCAT_LOOP_WAVE))
      return LoopChoice{kLoopWave, 1, s.P, 1, 1};
    const int rounds = (s.P + caps.cus - 1) / caps.cus;
    if (occ_regs >= 1) return LoopChoice{kLoopSolo, 1, s.P, 1, rounds < occ_regs ? rounds : occ_regs};
    if (caps.occ_stream >= 1) return LoopChoice{kLoopSolo, 0, s.P, 1, rounds < caps.occ_stream ? rounds : caps.occ_stream};
    return steps;
  }
  // Several slabs per problem: the workgroups of a launch poll each other and must all be resident.  The problems
  // are independent, so they may be split into groups that run one after the other (A: few enough per launch that
  // the keys stay in registers; B: as many as fit with the keys streamed every step).  Per step, A pays the
  // latency of a step once per group, B pays one more read of all keys: take the cheaper (7 us of step latency,
  // 6.5 TB/s of streaming rate: what the loop measures on this device).
  const int64_t cap_a = (int64_t)caps.cus * occ_regs, cap_b = (int64_t)caps.cus * caps.occ_stream;
  auto plan = [&](int64_t cap, int regs) {
    LoopChoice c = steps;
    const int64_t fit = cap / pl.nblk;                         // problems that fit at once
    if (fit < 1) return c;
    c.kind = kLoopResident;
    c.keys_in_regs = regs;
    c.launches = (int)((s.P + fit - 1) / fit);
    c.group = (s.P + c.launches - 1) / c.launches;             // balanced groups
    c.need = (int)(((int64_t)c.group * pl.nblk + caps.cus - 1) / caps.cus);
    return c;
  };
  const LoopChoice a = plan(cap_a, 1), b = plan(cap_b, 0);
  if (a.kind == kLoopSteps) return b;                          // (b may be kLoopSteps too)
  if (b.kind == kLoopSteps || a.launches <= b.launches) return a;
  const double es = s.dtype == WILDCAT_BF16 ? 2.0 : 4.0;
  const double key_read_us = (double)s.P * (double)s.n * s.d * es / 6.5e6;
  return (a.launches - b.launches) * 7.0 < key_read_us ? a : b;
}

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

Plan make_plan(const Shape &s) {
  Plan p = {};
  // Two keys per thread (16-byte history loads) once that still leaves >= 2 workgroups per compute unit.
  p.kpt = ((int64_t)s.P * s.n >= (int64_t)2 * kThreads * 512) ? 2 : 1;
  p.slab = kThreads * p.kpt;
  p.nblk = (int)((s.n + p.slab - 1) / p.slab);
  p.npad = (int64_t)p.nblk * p.slab;
  p.dpad = (s.d + kChunk - 1) / kChunk * kChunk;
  // Column statistics and packing: pieces of at least 128 keys, at most 512 per problem and about 2048 in all (with
  // many problems -- bins -- smaller pieces are workgroups that end before they have a second tile in flight).
  int64_t nb0 = (s.n + 127) / 128;
  const int64_t nb0_cap = 2048 / s.P > 1 ? 2048 / s.P : 1;
  nb0 = nb0 > 512 ? 512 : nb0;
  p.nb0 = (int)(nb0 > nb0_cap ? nb0_cap : nb0);
  // Gram pass: about 1024 workgroups in total, each a whole number of slabs; 512 for the matrix-core form (value
  // widths 64, 128, 256 at r > 16), which runs two workgroups per compute unit and whose partial sums cost a pass
  // of their own to add up, and for ranks up to 8 (k_gram_small8: two workgroups per compute unit as well; the
  // pass there is a few microseconds, and half as many, longer workgroups leave half as many partial sums).
  int rtiles = (s.r + 127) / 128;
  const bool gram_mfma = s.r > 16 && (s.dv == 64 || s.dv == 128 || s.dv == 256);
  int want = ((gram_mfma || s.r <= 8) ? 512 : 1024) / (s.P * rtiles);
  if (want < 1) want = 1;
  const int want_pieces = want;                              // (before the slab count caps it: k_gram_cols cuts inside the slab)
  if (want > p.nblk) want = p.nblk;
  p.slabs_per_chunk = (p.nblk + want - 1) / want;
  p.nchunk = (p.nblk + p.slabs_per_chunk - 1) / p.slabs_per_chunk;
  p.chunk_keys = (int64_t)p.slabs_per_chunk * p.slab;
  p.gram_cols = p.nblk == 1 && s.r <= 16 && s.n <= 256;
  if (p.gram_cols) {
    // Small bins of small rank (k_gram_cols: a thread per value column, no sums across threads): the bin is cut into
    // pieces of at least 16 keys, so that a few problems still spread over the device and no thread walks through
    // many keys; a workgroup takes 256 / (columns rounded up to a power of two >= 64) consecutive pieces.
    int tp = 64;
    while (tp < s.dv) tp <<= 1;
    const int pieces = want_pieces * (kThreads / tp);
    int64_t ck = (s.n + pieces - 1) / pieces;
    ck = (ck + 15) / 16 * 16;
    if (ck < 32 && s.n >= 32) ck = 32;                       // (every piece costs a partial result of r (d_v + 1) doubles)
    p.chunk_keys = ck;
    p.nchunk = (int)((s.n + ck - 1) / ck);
  }

  const size_t es = s.dtype == WILDCAT_BF16 ? 2 : 4;
  const size_t P = (size_t)s.P, n = (size_t)p.npad, r = (size_t)s.r, dv1 = (size_t)s.dv + 1;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  p.off_kbar = take(P * p.dpad * 8);
  p.off_kp = take(P * n * p.dpad * es);
  p.off_d0 = take(P * n * 8);
  p.off_p = take(2 * P * n * 8);
  p.off_bsum = take(P * r * p.nblk * 8);
  p.off_scal = take(P * 8 * 8);
  p.off_F = take(P * n * r * (s.history_f32 ? 4 : 8));
  p.off_L = take(P * r * r * 8);
  p.off_gpart = take(P * p.nchunk * r * dv1 * 8);
  p.off_g = take(P * r * dv1 * 8);
  p.off_mpart = take(P * p.nb0 * (size_t)p.dpad * 8);
  p.off_vminpart = take(P * p.nb0 * (size_t)s.dv * 4);
  p.off_vmaxpart = take(P * p.nb0 * (size_t)s.dv * 4);
  p.off_u = take(P * r * 8);
  p.off_sync = take(4);
  // pivot records of the resident loop (problems of several slabs only)
  p.off_mail = take(p.nblk > 1 ? P * mail_words(s.r, p.dpad) * 8 : 0);
  // Resident launches are an option for every loop of at least two steps (how many problems share a launch is
  // decided against the device, see choose_loop); a problem of one slab takes its single-launch form at any rank.
  p.persistent = p.nblk == 1 || s.r >= 2;
  p.total = off;
  return p;
}

}  // namespace wildcat

using namespace wildcat;

extern "C" int wildcat_version(void) { return 100; }

extern "C" const char *wildcat_strerror(int status) {
  switch (status) {
    case WILDCAT_OK: return "ok";
    case WILDCAT_EINVAL: return "invalid argument";
    case WILDCAT_EWORKSPACE: return "workspace missing, misaligned or too small";
    case WILDCAT_EHIP: return "HIP runtime call or kernel launch failed";
    case WILDCAT_EUNSUPPORTED: return "request not supported by this build";
    case WILDCAT_ETOOLARGE: return "shape exceeds the fixed size of the library's own scratch memory";
    default: return "unknown status";
  }
}

extern "C" size_t wildcat_workspace_bytes(int64_t n, int32_t d, int32_t r, const wildcat_opts *opts) {
  Shape s;
  if (resolve_shape(n, 0, d, r, opts, &s) != WILDCAT_OK || !bins_divide(s) || r / s.bins > kMaxRank) return 0;
  return make_plan(bin_view(s)).total;
}

static inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

extern "C" int wildcat_draw_uniforms(uint64_t seed, int64_t count, double *host_out) {
  if (count < 0 || (count > 0 && !host_out)) return WILDCAT_EINVAL;
  for (int64_t t = 0; t < count; ++t)
    host_out[t] = (double)(mix64(seed + (uint64_t)(t + 1) * 0x9E3779B97F4A7C15ull) >> 11) * 0x1.0p-53;
  return WILDCAT_OK;
}
