/*
 * libwildcat -- C ABI of the WildCat hot path for AMD MI355X (gfx950).
 *
 * WildCat ("WildCat: Near-Linear Attention in Theory and Practice") replaces
 * softmax attention over n keys by weighted softmax attention over a coreset
 * of r keys:
 *
 *   CompressKV (Alg. 2, with Alg. 1 "RPNys" inside) picks r pivot keys by
 *   randomly pivoted Nystrom on the kernel exp(beta <k,k'> / tau^2) of the
 *   recentred keys, and folds ALL n values into r rows with the Nystrom
 *   weights W = h(K_S,K_S)^-1 h(K_S,K):  V_S = W V,  w = W 1.
 *
 *   WtdAttn (Alg. 3) then evaluates, for every query q_i,
 *       A_is = exp(beta <q_i, k_s>),   O_i = (A V_S)_i / (A w)_i  if (A w)_i > 0 else 0,
 *   clipped column-wise to the value range [v_min, v_max] of Alg. 4.
 *
 * Conventions
 *   - Every tensor is dense, row-major, last index fastest:
 *       Q   [batch, q_heads,  m, d]        K [batch, kv_heads, n, d]
 *       V   [batch, kv_heads, n, dv]       out [batch, q_heads, m, dv]
 *     A "problem" is one (batch, kv_head) pair; P = batch * kv_heads.  Query
 *     head h attends to kv head h / (q_heads / kv_heads).
 *   - Unless marked HOST, every pointer is a DEVICE pointer on the current HIP
 *     device.  The caller owns every buffer, including the workspace; the
 *     library allocates and frees nothing, reads no environment variable and
 *     keeps no state between calls: every decision is a function of the
 *     arguments and of the current device's attributes, queried anew.  (One
 *     exception, stated there: wildcat_query_radius_static.)
 *   - All work is enqueued on opts->stream (NULL = the null stream).  No entry
 *     point synchronises with the host; results are valid once the stream has
 *     reached the end of the enqueued work.
 *   - Every function returning int returns WILDCAT_OK (0) or a negative
 *     wildcat_status.  Arguments are validated on the host before anything is
 *     launched: WILDCAT_EINVAL, WILDCAT_EWORKSPACE and WILDCAT_EUNSUPPORTED mean
 *     that nothing has been enqueued.  WILDCAT_EHIP (a launch or runtime call
 *     failed) may leave the kernels launched before the failure enqueued; the
 *     outputs are then unspecified.  No exception crosses the boundary.
 *     Non-finite inputs give unspecified (but memory-safe) results.
 *   - Calls that share a workspace or output buffers must be ordered by the
 *     caller (same stream, or events).
 *   - Sharing the device.  When wildcat_rpnys_single_launch() reports 1 for a
 *     shape with more than one slab of keys per problem, the selection loop of
 *     wildcat_compress_kv runs as launches whose workgroups wait for one
 *     another and therefore must all be resident at once.  The grid is sized
 *     for an otherwise idle device: such a call must not overlap other GPU
 *     work on the same device (another stream's kernels, a second
 *     wildcat_compress_kv), or its workgroups may hold part of the device while
 *     waiting for workgroups that cannot start.  The waits are bounded
 *     (opts->wait_limit): they then give up and the call reports r_eff = -1
 *     instead of hanging, but only after seconds.  A caller who shares the
 *     device sets opts->loop_driver = WILDCAT_LOOP_STEPS, which has no such
 *     requirement.  Every other kernel of the library may overlap anything.
 *   - The library depends on the HIP runtime (libamdhip64) and must use the
 *     same copy of it as the code that allocated the buffers and created the
 *     stream: a host program that ships its own runtime loads that first and
 *     this library afterwards.  On a second runtime in the process every
 *     launch fails (WILDCAT_EHIP).
 */
#ifndef WILDCAT_H
#define WILDCAT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { WILDCAT_F32 = 0, WILDCAT_BF16 = 1 } wildcat_dtype;

/* WILDCAT_HISTORY_F64 (default): every quantity that decides a pivot is float64, and the pivots
 * are those a float64 implementation of Alg. 1 draws from the same uniforms.
 * WILDCAT_HISTORY_F32 (fast mode): the history rows are stored in fp32, which halves the memory
 * traffic of the loop.  Each row is rounded before it is used, so the factorisation stays
 * consistent, but the residual diagonal differs from the float64 one by about 1e-7 relative:
 * pivots are still drawn from (that) residual by the same inverse-CDF rule, yet at large n some
 * differ from the float64 reference's.  Sums and the residual diagonal itself stay float64. */
typedef enum { WILDCAT_HISTORY_F64 = 0, WILDCAT_HISTORY_F32 = 1 } wildcat_history;

/* How wildcat_compress_kv launches the selection loop (Alg. 1).
 * WILDCAT_LOOP_AUTO: all steps in one launch per group of problems wherever the workgroups of a group can be
 *   resident on the device at once (see "Sharing the device" above), else one launch per step.
 * WILDCAT_LOOP_STEPS: always one launch per step; safe on a shared device, slower (the keys are re-read every
 *   step and every step pays a launch).
 * WILDCAT_LOOP_WAVE: like AUTO, but problems small enough for the wavefront-per-problem form (at most 128 keys --
 *   64 at d = 128 -- and 16 pivots per bin) take it whatever their number (AUTO takes it only when there are many);
 *   a tuning and testing switch.
 * All three draw the same pivots; results differ in the rounding of float64 sums only. */
typedef enum { WILDCAT_LOOP_AUTO = 0, WILDCAT_LOOP_STEPS = 1, WILDCAT_LOOP_WAVE = 2 } wildcat_loop;

typedef enum {
  WILDCAT_OK = 0,
  WILDCAT_EINVAL = -1,      /* null pointer, bad shape / dtype / option            */
  WILDCAT_EWORKSPACE = -2,  /* workspace missing, misaligned or too small          */
  WILDCAT_EHIP = -3,        /* a HIP runtime call or kernel launch failed          */
  WILDCAT_EUNSUPPORTED = -4, /* valid request that this build does not implement   */
  WILDCAT_ETOOLARGE = -5    /* shape beyond the fixed size of the library's own    */
                            /* scratch (wildcat_query_radius_static only)          */
} wildcat_status;

/* Options.  A zero-filled struct selects the paper's defaults. */
typedef struct {
  int32_t batch;     /* 0 -> 1                                                      */
  int32_t q_heads;   /* 0 -> kv_heads                                               */
  int32_t kv_heads;  /* 0 -> 1; q_heads must be a multiple (grouped-query attention)*/
  int64_t m;         /* queries per head; 0 -> n                                    */
  int32_t dv;        /* value width; 0 -> d                                         */
  int32_t dtype;     /* wildcat_dtype: storage type of Q, K, V, K_S and out         */
  double beta;       /* softmax scale of eq. (1); 0 -> 1/sqrt(d)                    */
  double rank_tol;   /* an entry of the residual diagonal p that drops to           */
                     /* <= rank_tol * its initial value is set to 0 (the key is     */
                     /* numerically in the span of the coreset).  0 -> 1e-10;       */
                     /* negative -> bare clamp max(p, 0).  See Alg. 1, last two     */
                     /* lines of the loop ("for numerical stability").              */
  const double *r_q; /* DEVICE [P] query radius R_Q per problem (input of Alg. 2).  */
                     /* Required by wildcat_compress_kv; fill it with               */
                     /* wildcat_query_radius or pass your own bound.                */
  const double *uniforms; /* DEVICE [P, r] pivot uniforms in [0,1), one per RPNys   */
                     /* step (a device pointer, like every array of this struct),   */
                     /* or NULL: then u[p, i] is element p*r+i of the stream        */
                     /* wildcat_draw_uniforms(seed, ...) documents.                 */
  int32_t bins;      /* B of Alg. 2 (Sec. 2.5); 0 -> 1.  Bin b is the contiguous block  */
                     /* of rows b n/B .. (b+1) n/B - 1 and gets r/B pivots, stored in  */
                     /* coreset slots b r/B ..; B must divide n and r (else EINVAL).   */
                     /* Only wildcat_compress_kv, wildcat_workspace_bytes and          */
                     /* wildcat_rpnys_single_launch act on it; wildcat_wtd_attn reads  */
                     /* every slot (ignores coreset.r_eff) when bins > 1.              */
  int32_t tau_length; /* sequence length in eq. (kernel-temperature) when bins > 1:    */
                     /* 0 -> the bin length n/B (the effective length Thm. 2 names),   */
                     /* 1 -> the full length n (Alg. 2 as printed)                     */
  int32_t history;   /* wildcat_history: precision in which the selection loop keeps   */
                     /* its history (the partial Cholesky rows it re-reads every step) */
  int32_t loop_driver; /* wildcat_loop: launch form of the selection loop                */
  void *stream;      /* hipStream_t                                                 */
  void *ev_loop_begin; /* optional hipEvent_t pair that wildcat_compress_kv records  */
  void *ev_loop_end; /* on the stream right before the first and right after the    */
                     /* last launch of the RPNys selection loop (for profiling)     */
  void *workspace;   /* device scratch, 256-byte aligned, of at least               */
  size_t workspace_bytes; /* wildcat_workspace_bytes(...) bytes                     */
  int64_t wait_limit; /* polls (about a microsecond each) after which a workgroup of the  */
                     /* resident selection loop stops waiting for another one; 0 ->      */
                     /* 2000000.  Negative: a hook for testing the give-up path -- every */
                     /* workgroup but the first of each problem leaves at once, the      */
                     /* first gives up at its first unanswered poll, and the call        */
                     /* reports r_eff = -1 (all kernels still end normally).  -2: the    */
                     /* same test for the second wait of a step: the workgroup that has  */
                     /* found the pivot leaves before handing it over, and the others    */
                     /* give up at their first unanswered poll for it.                   */
} wildcat_opts;

/* The compressed cache: output of CompressKV, input of WtdAttn.  All buffers are
 * caller-allocated device memory. */
typedef struct {
  int32_t *idx;   /* [P, r]  pivot index into the n keys, bin by bin in selection   */
                  /*         order; -1 in unused slots (a bin's rank was exhausted  */
                  /*         before its r/B pivots)                                 */
  int32_t *r_eff; /* [P, B]  number of pivots drawn in each bin (-1 in every entry: a    */
                  /*         wait inside the resident loop ran out, see "Sharing    */
                  /*         the device"; idx, k_s, v_s, w are then zero / -1 or    */
                  /*         unspecified, and wildcat_wtd_attn on them is memory-   */
                  /*         safe but meaningless)                                  */
  void *k_s;      /* [P, r, d]  storage dtype: original (un-recentred) key rows     */
  float *v_s;     /* [P, r, dv] W V                                                 */
  float *w;       /* [P, r]     W 1                                                 */
  float *v_min;   /* [P, dv]    column minima of V (Alg. 4, first line)             */
  float *v_max;   /* [P, dv]    column maxima of V                                  */
  double *tau;    /* [P, B]     temperature of each bin (eq. (kernel-temperature))  */
  void *v_t;      /* [P, dv, r64] fp16, r64 = r rounded up to a multiple of 64: the */
                  /*         MFMA operand form of V_S for bf16 storage,             */
                  /*           v_t[p, c, j] = fp16(v_s[p, j, c] / v_scale[p]),      */
                  /*         zero for j >= r.  fp16 rather than bf16 because Nystrom */
                  /*         weights have both signs: the sums of Alg. 3 cancel, and */
                  /*         8 significand bits are then too few.  Written by       */
                  /*         wildcat_compress_kv; after editing v_s by hand refresh */
                  /*         both with wildcat_pack_values.  NULL for fp32 storage. */
                  /*         If v_t or v_scale is NULL with bf16 storage, WtdAttn   */
                  /*         reads v_s instead, on the vector ALU (far slower).     */
  float *v_scale; /* [P]     power of two that keeps v_t inside fp16's range:       */
                  /*         2^(e - 14), e = exponent of max |v_s[p]| (1 if 0)      */
  double *W;      /* [P, B, r/B, n/B] or NULL.  For tests and debugging: if set,    */
                  /*         wildcat_compress_kv also writes the Nystrom weights    */
                  /*         themselves (Alg. 1's return value W = h(K_S,K_S)^-1     */
                  /*         h(K_S,K), per bin: the diagonal blocks of Alg. 2's W;  */
                  /*         zero rows in unused slots), which the method never     */
                  /*         needs as a matrix -- only V_S = W V and w = W 1 are    */
                  /*         used.  O(n r^2 / B^2) extra work per bin, one thread   */
                  /*         per key.  No other entry point reads it.               */
} wildcat_coreset;

/* Library version as major*10000 + minor*100 + patch. */
int wildcat_version(void);

/* Static text for a wildcat_status (never NULL). */
const char *wildcat_strerror(int status);

/* HOST.  Bytes of workspace wildcat_compress_kv needs for keys of length n, width
 * d, rank r under *opts (batch, kv_heads, dv, dtype, bins, history are read; opts may be NULL).
 * Returns 0 for invalid arguments.  wildcat_wtd_attn needs no workspace;
 * wildcat_query_radius can use one (see there). */
size_t wildcat_workspace_bytes(int64_t n, int32_t d, int32_t r, const wildcat_opts *opts);

/* HOST.  Fills host_out[0..count) with the library's pivot uniforms for `seed`:
 *   u_t = (mix64(seed + (t+1) * 0x9E3779B97F4A7C15) >> 11) * 2^-53,   t = 0, 1, ...
 * mix64 = the SplitMix64 output function.  The paper leaves the sampler of Alg. 1
 * ("s ~ p / sum p") open; this is the stream a bare seed stands for. */
int wildcat_draw_uniforms(uint64_t seed, int64_t count, double *host_out);

/* R_Q of Alg. 4: r_q_out[p] = max over the query rows of every query head that
 * shares kv head p of ||q||_2.  Q is [batch, q_heads, m, d] in opts->dtype.
 * r_q_out: device [P] doubles.  No workspace is required; if opts->workspace offers at
 * least 8 * (4096 + batch * q_heads) bytes (e.g. the workspace of the wildcat_compress_kv call
 * that follows on the same stream) it is used as scratch for per-workgroup maxima, which
 * is several times faster than the atomic updates of r_q_out used otherwise.  Same result. */
int wildcat_query_radius(const void *Q, int64_t m, int32_t d, const wildcat_opts *opts,
                         double *r_q_out);

/* The same result as wildcat_query_radius for callers that can neither allocate device memory nor offer a
 * workspace at this point -- code running under HIP graph capture, tight serving loops that compute R_Q for
 * new queries, harnesses that forbid allocation: the per-workgroup maxima go to a 64 KB array of device memory
 * that is part of the library's code object (each device the library runs on holds one copy until the process
 * ends; its address is looked up on the first call on a device and kept -- the one piece of state the library
 * has).  Allocates nothing, synchronises nothing, ignores opts->workspace.  Limit: batch * q_heads <= 4096, else
 * WILDCAT_ETOOLARGE and nothing is enqueued.  Nothing in the array needs clearing between calls (every entry a
 * call reads it has written itself), but all calls on a device share it: calls that may overlap on one device
 * (different streams) race and must be ordered by the caller.  Row widths that are not a power-of-two number
 * (<= 64) of 16-byte pieces take the atomic path of wildcat_query_radius, which uses no scratch at all. */
int wildcat_query_radius_static(const void *Q, int64_t m, int32_t d, const wildcat_opts *opts,
                                double *r_q_out);

/* CompressKV (Alg. 2) together with the value range of Alg. 4:
 *   kbar = row mean of K;  then for each of the B = opts->bins bins of rows:
 *   R_K = max_l ||k_l - kbar|| over the bin;  tau from eq. (kernel-temperature)
 *   with opts->r_q;  RPNys (Alg. 1) on the bin's recentred keys with kernel
 *   exp(beta <.,.> / tau^2) for r/B pivots, the pivot of the bin's step i drawn by
 *   inverse CDF from uniform u[p, b r/B + i]:  s = min{ l : sum_{l'<=l} p_l' > u * sum p };
 *   out->k_s = K[idx], out->v_s = W V, out->w = W 1 (W block diagonal over the bins:
 *   a bin's weights act on the bin's values), out->v_min/v_max, out->tau.
 * K [batch, kv_heads, n, d], V [batch, kv_heads, n, dv] in opts->dtype.
 * Requires 1 <= r <= n, d >= 1, opts != NULL with r_q and workspace set.
 * If a bin's residual mass reaches zero after r_eff < r/B pivots, its remaining slots
 * get idx = -1 and zero key, value and weight (they then add nothing in WtdAttn). */
int wildcat_compress_kv(const void *K, const void *V, int64_t n, int32_t d, int32_t r,
                        uint64_t seed, const wildcat_opts *opts, wildcat_coreset *out);

/* WtdAttn (Alg. 3): out[b, h, i, :] = clip( (A V_S)_i / (A w)_i  if (A w)_i > 0 else 0,
 * v_min, v_max ), A_is = exp(beta <q_i, k_s>), against the coreset of kv head
 * h / (q_heads / kv_heads).  Q [batch, q_heads, m, d], out [batch, q_heads, m, dv] in
 * opts->dtype; cs->idx and cs->tau are not read (cs->r_eff, if not NULL and opts->bins <= 1,
 * limits the slots that are read), so any (k_s, v_s, w, v_min, v_max) may be supplied -- e.g. all n keys with unit weights, which is exact
 * attention. */
int wildcat_wtd_attn(const void *Q, const wildcat_coreset *cs, void *out, int64_t m,
                     int32_t d, int32_t r, const wildcat_opts *opts);

/* HOST (queries the current device).  1 if wildcat_compress_kv will run the RPNys selection loop
 * (Alg. 1) of this shape with all steps inside one launch per group of problems -- either the key slabs of
 * the group's problems (bins) resident on the device at once, the workgroups of a problem synchronising
 * through memory, or, for problems of a single slab, one workgroup (one wavefront, if the problems are tiny
 * and many) alone with its problem -- and 0 if it will issue one launch per step; negative wildcat_status
 * for invalid arguments.  opts->loop_driver is honoured.  For profiling, reporting and the rule under
 * "Sharing the device". */
int wildcat_rpnys_single_launch(int64_t n, int32_t d, int32_t r, const wildcat_opts *opts);

/* HOST.  The launch form of the selection loop for a shape, as eight integers:
 *   out[0] driver: 0 one launch per step, 1 resident launches (slabs of a problem poll each other),
 *          2 one workgroup alone with each single-slab problem, 3 one wavefront per tiny problem
 *   out[1] keys per thread (1 or 2)       out[2] slabs (workgroups) per problem
 *   out[3] problems (bins) per launch     out[4] launches for all problems (driver 0: per step)
 *   out[5] 1 if the keys stay in registers for the whole loop, 0 if they are re-read every step
 *   out[6] workgroups a compute unit must hold during a launch     out[7] 0
 * With compute_units > 0 nothing touches a device: the plan is the one for a device with that many compute
 * units that can hold occ_resident_keys (0: cannot) resp. occ_streamed_keys workgroups of the loop kernel per
 * compute unit with the keys in registers resp. streamed.  With compute_units <= 0 the three figures are those
 * of the current device, and the plan is the one wildcat_compress_kv will use there. */
int wildcat_loop_plan(int64_t n, int32_t d, int32_t r, const wildcat_opts *opts, int32_t compute_units,
                      int32_t occ_resident_keys, int32_t occ_streamed_keys, int32_t out[8]);

/* Rewrites cs->v_t and cs->v_scale from cs->v_s (device buffers, see wildcat_coreset) for a coreset
 * of r rows and value width dv; batch and kv_heads are read from opts, whose dtype must
 * be WILDCAT_BF16.  For callers who assemble a coreset themselves instead of taking it
 * from wildcat_compress_kv (Alg. 3 accepts any weighted coreset). */
int wildcat_pack_values(const wildcat_coreset *cs, int32_t r, int32_t dv, const wildcat_opts *opts);

#ifdef __cplusplus
}
#endif
#endif /* WILDCAT_H */
