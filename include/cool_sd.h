/*
 * cool_sd.h -- C ABI of the MI355X (gfx950) verify-and-resample library for annealed
 * relaxed speculative decoding (Cool-SD).
 *
 * One call verifies, for a batch of B independent sequences, the L tokens a draft model Q
 * proposed against the target model P (Algorithm 1, verification stage):
 *
 *   p_i, q_i   softmax of the target / draft logits at draft position i = 1..L (+ bonus L+1)
 *   f_i        = min{1, omega_i p_i(x~_i) / q_i(x~_i)}, 0/0 := 1            (Eq. relax)
 *   accept_i   = [u_i <= f_i]
 *   tau        = number of positions before the first rejection              (Algorithm 1)
 *   x_{tau+1}  ~ G* = Norm([p - q f]_+) at the rejected position              (Theorem 2, Eq. opt_G)
 *                (or Norm([p - q]_+), Eq. g_tsd, in VANILLA mode),
 *                or ~ p_{L+1} when all L tokens were accepted                 (Algorithm 1, bonus)
 *   omega_i    relaxation schedule, e.g. delta * exp(-nu i - mu)              (Eq. sdar)
 *
 * Conventions
 *   - Pointers named *_dev are device pointers valid on the current HIP device; all others
 *     are host pointers.  The caller owns every buffer; the library allocates no device
 *     memory and never synchronises with the host: work is enqueued on the given stream.
 *   - Inputs are read-only; every output element is overwritten.
 *   - Functions return COOL_SD_OK (0) or a negative cool_sd_status.  Argument errors are
 *     detected on the host before anything is enqueued.  Draft tokens outside [0, V) are a
 *     contract violation that no status reports: wherever a token is used as an address the
 *     kernels clamp it into [0, V-1] first, so nothing outside the rows is read and the results
 *     are those of the clamped token.  COOL_SD_FLAG_CHECK_TOKENS (always on in the debug build
 *     libcool_sd_checked.so) marks such sequences with accept_len = next_token = -1.
 *   - Logits must be finite or -inf (-inf = token excluded); every row needs at least one
 *     finite logit.  Uniforms lie in [0, 1).
 *   - The workspace holds only intermediate results of one call (chunk statistics, masses);
 *     nothing persists between calls and it needs no initialisation.  Calls that share a
 *     workspace must be ordered on one stream.
 *   - No kernel spins or waits on another workgroup.  The only global atomics are integer counts
 *     whose sums do not depend on the order (top-k on rows beyond 65536 logits) and a per-sequence
 *     ticket that decides which workgroup finishes a sequence, not what it computes; for given
 *     inputs the outputs are bit-identical from run to run.
 */
#ifndef COOL_SD_H
#define COOL_SD_H

#include <stddef.h>
#include <stdint.h>

/* The library is built with hidden visibility; these are its only exported symbols. */
#if defined(__GNUC__) || defined(__clang__)
#define COOL_SD_API __attribute__((visibility("default")))
#else
#define COOL_SD_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { COOL_SD_F32 = 0, COOL_SD_BF16 = 1 } cool_sd_dtype;

typedef enum {
  COOL_SD_SCHED_UNIFORM = 0, /* omega_i = delta                         (uniform relaxation)   */
  COOL_SD_SCHED_EXP = 1,     /* omega_i = delta exp(-nu i - mu)          (Eq. sdar)             */
  COOL_SD_SCHED_LINEAR = 2   /* omega_i ~ (ell - i), normalised to sum delta L (App., schedule ablation) */
} cool_sd_sched;

typedef enum {
  COOL_SD_RESAMPLE_OPT = 0,     /* G* = Norm([p - min(q, omega p)]_+)       (Eq. opt_G) */
  COOL_SD_RESAMPLE_VANILLA = 1, /* G^van = Norm([p - q]_+)                  (Eq. g_tsd) */
  COOL_SD_RESAMPLE_LANTERN = 2  /* Norm([P^{k,lambda} - q]_+)               (Eq. g_lantern);
                                   cool_sd_verify_lantern only */
} cool_sd_resample_mode;

typedef enum {
  COOL_SD_OK = 0,
  COOL_SD_EINVAL = -1,       /* null pointer, bad shape / stride / dtype / option           */
  COOL_SD_EWORKSPACE = -2,   /* workspace missing, misaligned or smaller than required       */
  COOL_SD_ELAUNCH = -3,      /* the HIP runtime refused a launch                             */
  COOL_SD_EUNSUPPORTED = -4, /* valid request the kernels do not implement (none at present)  */
  COOL_SD_ETOOLARGE = -5     /* cool_sd_verify_noalloc: the shape needs more workspace than
                                COOL_SD_NOALLOC_WORKSPACE_BYTES                                  */
} cool_sd_status;

/* Options of cool_sd_verify (cool_sd_params.flags). */
typedef enum {
  /* Algorithm 1 stops at the first rejection; with this flag so does the memory traffic.  Two
   * forms, chosen by the shape (cool_sd_early_exit_form tells which):
   *   V <= 16384 (and L <= 1024, 16-byte aligned rows: base pointers and strides multiples of 16
   *   bytes, V a multiple of 8 for bf16 / 4 for fp32): one workgroup per sequence walks positions
   *   1, 2, ... and reads no row pair after the rejected one (except the single pair whose loads
   *   were already issued ahead); the workspace is not touched.  Pays when B is at least the
   *   number of compute units.
   *   16384 < V <= 524288, any alignment: the call verifies in rounds of 1, 1, 2, 4, ... positions
   *   (two launches per round); a sequence's rows are read up to the end of the round that holds
   *   its rejection, then the row pair it samples from once more.  Pays when rejections come
   *   early in the window; costs about 7 us per round when they do not.
   * Not honoured under top-k, by cool_sd_verify_lantern and cool_sd_verify_diagnostics, or for
   * shapes outside the two forms: the call then reads every row, and cool_sd_early_exit_form
   * returns COOL_SD_EARLY_EXIT_NONE.
   * When honoured, p_tok / q_tok / f of positions after the rejected one are NaN.  accept_len,
   * next_token and resid_mass mean the same in all forms. */
  COOL_SD_FLAG_EARLY_EXIT = 1,
  /* Checked mode of the verify calls: one more (small) kernel after the others looks at every
   * draft token on the device; a sequence that holds a token outside [0, V) gets
   * accept_len = -1, next_token = -1 and resid_mass = 0 instead of the results of the clamped
   * token.  Every kernel still runs to its end on such input.  The debug build of the library
   * (libcool_sd_checked.so, compiled with -DCOOL_SD_CHECKED_BUILD) behaves as if every call set
   * this bit. */
  COOL_SD_FLAG_CHECK_TOKENS = 2,
  /* The draw x ~ G* (or ~ p for the bonus / draft-side draw) is made in fp32 and re-done in fp64
   * only where fp32 cannot resolve the law: its total mass below 1/16 (p and q f nearly cancel),
   * or the levels of the fp32 search disagreeing by rounding.  With this bit every draw of the
   * call takes the fp64 path -- for validation; several times slower per sequence.  Results: the
   * same token except where u lies within ~1e-7 of a boundary of the law's CDF. */
  COOL_SD_FLAG_EXACT_DRAW = 4
} cool_sd_flags;

typedef struct {
  int32_t B;             /* sequences, >= 1                                                   */
  int32_t L;             /* draft length, 1..4096                                             */
  int32_t V;             /* vocabulary size, >= 1; rows of V contiguous elements              */
  int32_t dtype;         /* cool_sd_dtype of every logit tensor                               */
  int64_t t_stride_b;    /* element strides of the target logits [B, L(+1), V]                */
  int64_t t_stride_l;
  int64_t d_stride_b;    /* element strides of the draft logits [B, L, V]                     */
  int64_t d_stride_l;
  int64_t omega_stride_b;/* 0: omega is [L], shared by all sequences; else omega is [B, L]
                            with this element stride between sequences                        */
  int32_t has_bonus;     /* 1: target holds L+1 rows per sequence; 0: L rows, no bonus token  */
  int32_t top_k;         /* 0 = off; else 1..V: keep logits >= the k-th largest of the row
                            (ties kept), on BOTH models, after guidance and temperature.
                            Rows of at most 65536 logits are selected inside the statistics
                            kernel; longer rows by three radix passes over the row first     */
  float cfg_scale;       /* s of l = l_u + s (l_c - l_u); used iff the *_uncond pointers are
                            given (classifier-free guidance, App. implementation details)     */
  float temperature;     /* > 0; logits are multiplied by fl32(1/temperature); 1 = off        */
  int32_t resample_mode; /* cool_sd_resample_mode                                             */
  int32_t flags;         /* bit set of cool_sd_flags; unknown bits are an error                */
} cool_sd_params;

/* Relaxation schedule (Eq. sdar and the uniform / linear variants), host only, O(L).
 * kind: cool_sd_sched.  param: nu (EXP, > 0), ell (LINEAR, >= L), ignored (UNIFORM).
 * omega_out: host float[L]; omega_out[i-1] = omega_i of the paper.  Evaluated in fp64 and
 * rounded once to fp32.  COOL_SD_EINVAL on bad arguments (LINEAR with ell < L would need a
 * negative weight). */
COOL_SD_API int cool_sd_schedule(int32_t kind, int32_t L, float delta, float param, float* omega_out);

/* Bytes of device workspace cool_sd_verify / cool_sd_verify_lantern / cool_sd_verify_diagnostics /
 * cool_sd_resample / cool_sd_diagnostics need for these params
 * (for resample only B, V, dtype and top_k matter).  0 on invalid params. */
COOL_SD_API size_t cool_sd_workspace_bytes(const cool_sd_params* p);

/* Zero a workspace on the stream.  Optional (no call depends on the workspace's contents);
 * kept for callers that want defined memory.  workspace_dev must be 256-byte aligned. */
COOL_SD_API int cool_sd_workspace_init(void* workspace_dev, size_t workspace_bytes, void* hip_stream);

/* Verification stage of Algorithm 1 for B sequences; asynchronous on hip_stream.
 *   target_dev          [B, L + has_bonus, V] logits of P (conditional ones under guidance)
 *   target_uncond_dev   same shape/strides, or NULL (no guidance)
 *   draft_dev           [B, L, V] logits of Q;  draft_uncond_dev likewise (both or neither)
 *   draft_tokens_dev    [B, L] int32, contiguous: x~_i
 *   omega_dev           float [L] (or [B, L], see omega_stride_b), >= 0
 *   u_accept_dev        float [B, L]: the uniforms r_i of Algorithm 1
 *   u_resample_dev      float [B]: drives the draw from G* / the bonus draw (inverse CDF in
 *                       ascending token order: smallest k with g(0)+..+g(k) > u R)
 *   accept_len_dev      out int32 [B]: tau in [0, L]
 *   next_token_dev      out int32 [B]: x_{tau+1}; -1 iff tau == L and has_bonus == 0
 *   p_tok_dev, q_tok_dev, f_dev   out float [B, L], each optional (NULL = skip):
 *                       p_i(x~_i), q_i(x~_i), f_i for every position (also after tau; but see
 *                       COOL_SD_FLAG_EARLY_EXIT)
 *   resid_mass_dev      out float [B], optional: R = sum_x g(x) of the sampled law
 *                       (sum of p for the bonus draw, 0 when next_token = -1)
 * The accepted tokens are draft_tokens[b, 0:tau]; they are not copied. */
COOL_SD_API int cool_sd_verify(const cool_sd_params* p,
                   const void* target_dev, const void* target_uncond_dev,
                   const void* draft_dev, const void* draft_uncond_dev,
                   const int32_t* draft_tokens_dev,
                   const float* omega_dev,
                   const float* u_accept_dev,
                   const float* u_resample_dev,
                   int32_t* accept_len_dev,
                   int32_t* next_token_dev,
                   float* p_tok_dev, float* q_tok_dev, float* f_dev,
                   float* resid_mass_dev,
                   void* workspace_dev, size_t workspace_bytes,
                   void* hip_stream);

/* cool_sd_verify for callers that can neither allocate device memory nor carry a workspace: code
 * under HIP graph capture with a fixed set of buffers, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, kernels and results as cool_sd_verify, without the workspace
 * arguments: the intermediate results of the call (chunk statistics, per-sequence statistics, chunk
 * masses) live in a device array inside the library, COOL_SD_NOALLOC_WORKSPACE_BYTES large, of
 * which every GPU the library is used on holds one copy until the process ends.  The call
 * allocates nothing and frees nothing.
 *   - Shapes whose workspace (what cool_sd_verify itself would use for these params) exceeds the
 *     array are refused with COOL_SD_ETOOLARGE before anything is enqueued; the five benchmark
 *     configurations fit (the largest, B=128 L=8 V=262144, uses 0.6 MB).
 *   - All calls on one GPU share that GPU's array, whatever their stream: two calls that overlap
 *     in time on one GPU race.  Order them (one stream, or events).  Nothing in the array needs
 *     initialisation and nothing in it is meaningful after the call.
 *   - The array's device address is looked up at the first call on each device (not a stream
 *     operation, no allocation); make that first call outside a stream capture. */
#define COOL_SD_NOALLOC_WORKSPACE_BYTES (4u << 20)
COOL_SD_API int cool_sd_verify_noalloc(const cool_sd_params* p,
                                       const void* target_dev, const void* target_uncond_dev,
                                       const void* draft_dev, const void* draft_uncond_dev,
                                       const int32_t* draft_tokens_dev,
                                       const float* omega_dev,
                                       const float* u_accept_dev,
                                       const float* u_resample_dev,
                                       int32_t* accept_len_dev,
                                       int32_t* next_token_dev,
                                       float* p_tok_dev, float* q_tok_dev, float* f_dev,
                                       float* resid_mass_dev,
                                       void* hip_stream);

/* Verification stage of Algorithm 1 with the acceptance probability of the LANTERN family in
 * place of Eq. relax (the paper's comparison system, Eq. p_lantern / Eq. f_lantern, and its
 * ablation "LANTERN++ with G*"):
 *   A(x~_i)  = {x~_i} and the longest prefix n_1..n_m of x~_i's neighbour list, nearest first,
 *              with p_i(n_1) + ... + p_i(n_m) < lambda p_i(x~_i)
 *   f_i      = min{1, sum_{y in A(x~_i)} p_i(y) / q_i(x~_i)}, 0/0 := 1          (Eq. f_lantern)
 * and x_{tau+1} drawn, by p->resample_mode, from
 *   OPT      G* of Eq. opt_G for this f.  Because f_i >= f_i^van, G* equals Norm([p - q]_+)
 *            (Proposition on the design of G), which is what is evaluated;
 *   VANILLA  Norm([p - q]_+)                                                    (Eq. g_tsd)
 *   LANTERN  Norm([P^{k,lambda} - q]_+): the probability of A(x~_{tau+1}) moved onto x~_{tau+1}
 *            (Eq. p_lantern, Eq. g_lantern).
 *   neighbors_dev  int32 [V, k], row x = the k nearest neighbours of token x in the codebook's
 *                  latent space, nearest first; entries < 0, >= V or equal to x are skipped;
 *                  the remaining entries of a row must be distinct.  1 <= k <= 65536
 *   lambda         >= 0, finite
 *   p_agg_dev      out float [B, L], optional: sum_{y in A(x~_i)} p_i(y)
 *   count_dev      out int32 [B, L], optional: m, the neighbours taken into A(x~_i)
 * Everything else as in cool_sd_verify (there is no omega; COOL_SD_FLAG_EARLY_EXIT is ignored).
 * The set is decided from fp32 weights p_i(n)/p_i(x~_i); a running sum within rounding of
 * lambda may fall on either side. */
COOL_SD_API int cool_sd_verify_lantern(const cool_sd_params* p,
                           const void* target_dev, const void* target_uncond_dev,
                           const void* draft_dev, const void* draft_uncond_dev,
                           const int32_t* draft_tokens_dev,
                           const int32_t* neighbors_dev, int32_t k, float lambda,
                           const float* u_accept_dev,
                           const float* u_resample_dev,
                           int32_t* accept_len_dev,
                           int32_t* next_token_dev,
                           float* p_tok_dev, float* q_tok_dev, float* f_dev,
                           float* resid_mass_dev,
                           float* p_agg_dev, int32_t* count_dev,
                           void* workspace_dev, size_t workspace_bytes,
                           void* hip_stream);

/* Stand-alone resampling step (Eq. opt_G / Eq. g_tsd): one (target, draft) row pair per
 * sequence.  p->L, strides_l and has_bonus are ignored; rows are [B, V] with element strides
 * t_stride_b / d_stride_b.  omega_rows_dev float [B], u_dev float [B].
 * draft_rows_dev == NULL samples from p itself: the bonus draw of Algorithm 1, and, with the
 * draft model's logits passed as "target", the drafting loop's draw x~ ~ q (guidance,
 * temperature and top-k apply as configured).
 *   token_dev out int32 [B], resid_mass_dev out float [B] (optional; the mass of the law that
 *   was sampled: R of Eq. opt_G / Eq. g_tsd, 1 when the law is p itself).
 * Rows of at most 16384 logits (32768 when 16-byte aligned) are served by a single kernel launch
 * (except truncated rows with a draft), so a call per drafted token costs one launch latency; so
 * are draft-less truncated rows of up to 65536 logits (bf16) or 32768 (fp32). */
COOL_SD_API int cool_sd_resample(const cool_sd_params* p,
                     const void* target_rows_dev, const void* target_uncond_rows_dev,
                     const void* draft_rows_dev, const void* draft_uncond_rows_dev,
                     const float* omega_rows_dev, const float* u_dev,
                     int32_t* token_dev, float* resid_mass_dev,
                     void* workspace_dev, size_t workspace_bytes,
                     void* hip_stream);

/* Per-position diagnostics of Theorem 2 for the drafted prefix, asynchronous on hip_stream:
 *   alpha_dev out float [B, L]:  alpha_i = sum_x min{q_i(x), omega_i p_i(x)} = sum_x q_i(x) f_i(x),
 *             the probability that position i accepts a token drawn from q_i; the expected
 *             accepted length is 1 + sum_i prod_{j<=i} alpha_j averaged over drafts (Eq. token_exp)
 *   beta_dev  out float [B, L]:  beta_i = sum_x [min{q_i(x), omega_i p_i(x)} - p_i(x)]_+, half of
 *             what position i adds to the total-variation bound when G* resamples
 *             (Theorem 2, proof Step 2: sum|p - q f| - sum(1-f)q = 2 beta); 0 iff omega_i <= 1
 *             or the excess vanishes, so strict speculative decoding reports all zeros.
 * Tensors, strides, omega and the logit transform are those of cool_sd_verify (the bonus row of
 * the target tensor is not read); resample_mode is ignored.  Same workspace, same size.  Rows
 * of at most 16384 logits without top-k are read once; otherwise twice (statistics, then sums). */
COOL_SD_API int cool_sd_diagnostics(const cool_sd_params* p,
                        const void* target_dev, const void* target_uncond_dev,
                        const void* draft_dev, const void* draft_uncond_dev,
                        const float* omega_dev,
                        float* alpha_dev, float* beta_dev,
                        void* workspace_dev, size_t workspace_bytes,
                        void* hip_stream);

/* cool_sd_verify and cool_sd_diagnostics in one call (Algorithm 1's verification stage plus the
 * per-position terms of Theorem 2 for the same relaxation): same arguments and results as the
 * two calls, alpha_dev / beta_dev required.  For rows of at most 16384 logits without top-k every
 * logit is read ONCE for both (the workgroup that holds a row pair leaves its softmax statistics,
 * the logits of x~_i, alpha_i and beta_i; the per-sequence kernel follows), so that a caller who
 * tunes delta online against a total-variation budget pays no second pass; otherwise the
 * diagnostics pass follows the verify call's kernels on the stream and reuses the row statistics
 * and top-k thresholds they left in the workspace (the logits are read twice, not three times).
 * COOL_SD_FLAG_EARLY_EXIT is ignored (the diagnostics need every row). */
COOL_SD_API int cool_sd_verify_diagnostics(const cool_sd_params* p,
                               const void* target_dev, const void* target_uncond_dev,
                               const void* draft_dev, const void* draft_uncond_dev,
                               const int32_t* draft_tokens_dev,
                               const float* omega_dev,
                               const float* u_accept_dev,
                               const float* u_resample_dev,
                               int32_t* accept_len_dev,
                               int32_t* next_token_dev,
                               float* p_tok_dev, float* q_tok_dev, float* f_dev,
                               float* resid_mass_dev,
                               float* alpha_dev, float* beta_dev,
                               void* workspace_dev, size_t workspace_bytes,
                               void* hip_stream);

/* How cool_sd_verify (and cool_sd_verify_noalloc) would honour COOL_SD_FLAG_EARLY_EXIT for these
 * parameters.  rows_aligned: nonzero when every logit row of the call starts on a 16-byte boundary
 * (base pointers and strides) and V is a multiple of a 16-byte vector.  Host only: no device call.
 * Returns one of the values below, or COOL_SD_EINVAL. */
#define COOL_SD_EARLY_EXIT_NONE 0     /* flag clear or not honoured: every row is read        */
#define COOL_SD_EARLY_EXIT_SEQUENCE 1 /* one workgroup per sequence, position by position     */
#define COOL_SD_EARLY_EXIT_ROUNDS 2   /* long rows: rounds of positions                       */
COOL_SD_API int cool_sd_early_exit_form(const cool_sd_params* p, int rows_aligned);

/* Static description of a cool_sd_status. */
COOL_SD_API const char* cool_sd_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* COOL_SD_H */
