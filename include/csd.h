/*
 * csd.h - C ABI of the MI355X (gfx950) hot path of continuous speculative
 * decoding for autoregressive image generation (arxiv 2411.11925).
 *
 * The boundary follows the paper's statement of one speculative step (Alg. 1):
 * the conditioning vectors that the draft model M_q and the target model M_p
 * produce for gamma draft positions go in; the accepted-prefix length n and the
 * tokens [x_1..x_n, x'] come out.  Everything in between runs in HIP kernels of
 * this library: the T-step reverse diffusion of both heads on one aligned
 * trajectory (shared reparameterisation noise eps_t, Sec. 3.2 and App. A.2),
 * log Sigma of Eq. 6, the accept test of Eq. 7 / Alg. 1, and acceptance-rejection
 * resampling from max(0,p-q)/Z with the threshold of Corollary 1 (Sec. 3.3).
 *
 * Conventions
 *   - "device" pointers are HIP device memory on the head's device, owned by the
 *     caller; "host" pointers are ordinary host memory.  The library owns only
 *     what csd_init_head allocates (freed by csd_free_head).
 *   - All matrices are row-major.  A row is one (image, draft position) pair;
 *     group g holds rows g*gamma .. g*gamma+gamma-1; R = n_groups*gamma.
 *   - `hip_stream` is a hipStream_t (NULL = the default stream).  Calls enqueue
 *     work and return; outputs are valid once the stream has been synchronised.
 *     No call synchronises the device except csd_init_head / csd_free_head.
 *   - Every function returning int gives 0 (CSD_OK) or a negative CSD_E* code;
 *     csd_last_error() then holds a message (thread-local).  Nothing aborts.
 *   - Calls may be enqueued on different streams (default priority) from one host
 *     thread and then run side by side, each with a workspace of its own: e.g. the
 *     bonus sample for position gamma+1 beside the target call of a verify window.
 *     Calls that run both heads (csd_denoise_lockstep, csd_denoise_ablation) and
 *     single-head calls of 8192 rows or more also use the library's own side streams
 *     of the device; these are shared, so two such calls are correct together but
 *     share those streams.  Heads are read-only after csd_init_head /
 *     csd_set_guidance and may serve any number of calls at once.
 *   - Random numbers come from Philox-4x32-10 keyed by `seed` and countered by
 *     the GLOBAL row index row_offset + r, so a workload may be split over
 *     calls (or devices) without changing any result.
 */
#ifndef CSD_H
#define CSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CSD_OK            0
#define CSD_EINVAL       (-1)  /* bad argument: null pointer, shape or size out of range */
#define CSD_ENOMEM       (-2)  /* host or device allocation failed */
#define CSD_EHIP         (-3)  /* a HIP runtime call failed */
#define CSD_EUNSUPPORTED (-4)  /* valid request that this build does not implement */

#define CSD_F32   0            /* GEMMs in fp32 (vector FMA) */
#define CSD_BF16  1            /* GEMMs on bf16 MFMA with fp32 accumulation */

#define CSD_COSINE 0           /* native T-step cosine schedule, betas clipped at 0.999 */
#define CSD_TABLE  1           /* caller supplies alpha_bar[0..T] */

/* The head's sampler: the Gaussian p(x_{t-1}|x_t) of one reverse step (appendix "More
 * variants of diffusion model": any sampler with an explicit step density fits).
 * DDPM: Eq. 3 with the learned-range variance (definition below).
 * DDIM: mu = sqrt(abar_{t-1}) x0_hat + sqrt(max(0, 1-abar_{t-1}-sigma_t^2)) eps_hat with
 *       x0_hat = (x_t - sqrt(1-abar_t) eps_hat)/sqrt(abar_t) and the fixed variance
 *       sigma_t^2 = eta^2 beta~_t (beta~_1 := beta~_2, so the final step keeps a density);
 *       the head's v output is not used; eta = 1 is the DDPM posterior. */
#define CSD_SAMPLER_DDPM 0
#define CSD_SAMPLER_DDIM 1

#define CSD_TIME_FEATURES 256  /* sinusoidal features of the step index */

/* streams of the counter-based generator (third counter word = slot | stream << 16) */
#define CSD_STREAM_TRAJ        0  /* slot T: x_T; slot t-1: eps_t of the step t -> t-1 */
#define CSD_STREAM_ACCEPT_U    1  /* slot 0: the uniform r_i of the accept test */
#define CSD_STREAM_RESAMPLE_N  2  /* slot k: proposal noise of resampling trial k */
#define CSD_STREAM_RESAMPLE_U  3  /* slot k: uniform of resampling trial k */
#define CSD_STREAM_BONUS       4  /* trajectory noise of the target-only sample for position gamma+1;
                                    its "row" is the global GROUP index */
#define CSD_STREAM_TRAJ_P      5  /* the target's own x_T and eps_t when the two paths are not aligned
                                    (csd_denoise_ablation, CSD_RATIO_UNALIGNED); slots as in stream 0 */
#define CSD_STREAM_GMM_PICK    6  /* mixture heads: the uniform that picks a component; slot 0: the draft's
                                    sample, slot 1+k: resampling trial k */

/* how csd_denoise_ablation forms the path ratio before the final step (Table 1) */
#define CSD_RATIO_ALIGNED      0  /* p(Y_p)/q(Y_q) with eps^p_t = eps^q_t (Sec. 3.2): the method */
#define CSD_RATIO_UNALIGNED    1  /* p(Y_p)/q(Y_q) with independent noise in the two paths (Eq. 4 alone) */
#define CSD_RATIO_SINGLE_PATH  2  /* p(Y)/q(Y), both densities on the draft's path (Eq. 2) */

/* bits of flags[g] written by csd_resample */
#define CSD_FLAG_CAP        1u    /* max_trips reached; the last proposal was emitted */
#define CSD_FLAG_NONFINITE  2u    /* a NaN log-ratio was met and treated as "do not accept" */

typedef struct csd_head csd_head_t;   /* opaque; immutable after csd_init_head */

/*
 * One diffusion head: (eps_hat, v) = Head(x_t, t, z).  The paper leaves the
 * network open ("a neural network with parameter theta", Sec. 3.1); this
 * library implements an adaLN-modulated residual MLP:
 *   E_t  = Lin_t2(SiLU(Lin_t1(sincos_256(t_scale*(t-1)))))      (per step, at init)
 *   e    = Lin_cond(z);  s = SiLU(E_t + e);  h = Lin_in(x_t)
 *   L x : (shift,scale,gate) = Lin_mod_l(s);  u = LN(h)*(1+scale)+shift;
 *         h += gate * Lin_fc2_l(SiLU(Lin_fc1_l(u)))
 *   (shift,scale) = Lin_fmod(s);  o = Lin_out(LN(h)*(1+scale)+shift)   in R^{2D}
 *   eps_hat = o[0:D] + eps_skip_gain*sqrt(1-abar_t)*x_t ;  v = o[D:2D]
 * LN has no affine part and uses the biased variance.  The reverse transition
 * (Eq. 3) is N(mu_t, diag sigma_t^2) with
 *   mu_t = (x_t - beta_t/sqrt(1-abar_t)*eps_hat)/sqrt(alpha_t),
 *   log sigma_t^2 = f*log(beta_t) + (1-f)*log(beta~_t), f=(v+1)/2, beta~_1 := beta~_2.
 *
 * Packed weight order (fp32, each matrix [out,in] row-major, bias after matrix):
 *   t1[W,256] t2[W,W] cond[W,C] in[W,D] { mod_l[3W,W] fc1_l[W,W] fc2_l[W,W] }xL
 *   fmod[2W,W] out[2D,W]
 * Limits: token_dim in {4,8,16}; width a multiple of 64, <= 4096; cond_dim a
 * multiple of 8; 1 <= n_blocks <= 64; 1 <= n_steps <= 4096.
 */
typedef struct {
    int32_t token_dim;       /* D */
    int32_t cond_dim;        /* C */
    int32_t width;           /* W */
    int32_t n_blocks;        /* L */
    int32_t n_steps;         /* T */
    int32_t gemm_dtype;      /* CSD_F32 | CSD_BF16 */
    int32_t schedule;        /* CSD_COSINE | CSD_TABLE */
    int32_t sampler;         /* CSD_SAMPLER_DDPM (0) | CSD_SAMPLER_DDIM */
    const double* alpha_bar; /* host [n_steps+1], alpha_bar[0]=1, strictly decreasing; CSD_TABLE only */
    float ln_eps;            /* <= 0 selects 1e-6 */
    float t_scale;           /* <= 0 selects 1000/T */
    float eps_skip_gain;     /* 0 = plain eps-prediction */
    float ddim_eta;          /* CSD_SAMPLER_DDIM: sigma_t^2 = eta^2 beta~_t, eta > 0; else must be 0 */
} csd_head_cfg_t;

/* Number of fp32 values in the packed weight blob of `cfg`, 0 if cfg is invalid. */
size_t csd_param_count(const csd_head_cfg_t* cfg);

/*
 * Copies and packs `weights_host` (host, csd_param_count(cfg) floats; the
 * caller keeps its blob) onto HIP device `device`, computes the schedule
 * constants and the time-embedding table there, and returns the head in *out.
 * Synchronises `device`.  Errors: CSD_EINVAL (limits above, n_floats mismatch,
 * bad alpha_bar), CSD_ENOMEM, CSD_EHIP.
 */
int csd_init_head(const csd_head_cfg_t* cfg, const float* weights_host, size_t n_floats,
                  int device, csd_head_t** out);

/* Frees the head's device and host memory (NULL is allowed).  Synchronises its device. */
void csd_free_head(csd_head_t* head);

/*
 * Classifier-free guidance for this head (the paper's runs use it, Sec. 4 and the appendix
 * on guidance scale; how it enters the head is not spelled out there).  Reading taken: while
 * enabled, every conditioning array passed for this head holds TWO vectors per row, [R, 2, C]
 * = (conditional, unconditional); each step evaluates the head with both on the same x_t and
 *   eps_hat = eps_u + scale (eps_c - eps_u),   v = v_c.
 * The guided head is still one Gaussian step, so everything downstream is unchanged.
 * scale = 1 is the conditional head.  Workspace needs grow (csd_workspace_bytes accounts for
 * it).  A setting, not per-call state: do not change it while calls on this head are in flight.
 */
int csd_set_guidance(csd_head_t* head, int32_t enabled, float scale);

/*
 * Bytes of device workspace csd_denoise_lockstep / csd_head_eval need for
 * n_rows rows with these heads (either head may be NULL).  0 on invalid input.
 */
size_t csd_workspace_bytes(const csd_head_t* draft, const csd_head_t* target, int64_t n_rows);

/*
 * Lockstep denoising on the aligned trajectory (Sec. 3.2; App. A.2; Alg. 1,
 * "keep the eps_t the same").  For each row r: x_T^q = x_T^p = eps_T, then for
 * t = T..1 both heads take x_{t-1} = mu_t + temperature*sigma_t*eps_t with the
 * same eps_t, and for t = T..2 the row accumulates
 *   log Sigma += 1/2 sum_d (log sigma^2_{q,t,d} - log sigma^2_{p,t,d})   (Eq. 6).
 * Output summary [R, 5D+1] fp32 (device):
 *   [ mu^p_1 | log sigma^2_{p,1} | mu^q_1 | log sigma^2_{q,1} | x_0 | log Sigma ]
 * where x_0 = mu^q_1 + temperature*sigma_{q,1}*eps_1 is the draft token (Eq. 7).
 * z_q, z_p: device [R, C] fp32 conditioning vectors of M_q and M_p.
 * Both heads must share token_dim, n_steps and device; `workspace` is device
 * memory of at least csd_workspace_bytes(draft,target,R) bytes, 256-byte
 * aligned, free for other use once the stream has passed this call.
 * n_groups = 0 is a no-op.  Errors: CSD_EINVAL, CSD_EHIP.
 */
int csd_denoise_lockstep(const csd_head_t* draft, const csd_head_t* target,
                         const float* z_q, const float* z_p,
                         int64_t n_groups, int32_t gamma,
                         uint64_t seed, uint64_t row_offset, float temperature,
                         float* summary, void* workspace, size_t workspace_bytes,
                         void* hip_stream);

/*
 * The comparison of ratio calculations (Table 1; the appendix on the approximation of
 * the ratio) and the alignment ablation (the table of acceptance rate and token
 * distance with and without alignment; Theorem 1).  Same arguments, layout and
 * errors as csd_denoise_lockstep, plus:
 *   ratio_mode  CSD_RATIO_ALIGNED: the lockstep path itself (the summary is bit-identical
 *               to csd_denoise_lockstep's).  CSD_RATIO_UNALIGNED: the target draws its own
 *               x_T^p and eps^p_t (stream CSD_STREAM_TRAJ_P); the exponents of the Gaussian
 *               densities (Eq. 3) no longer cancel and are accumulated.  CSD_RATIO_SINGLE_PATH:
 *               the target head is evaluated at the draft's x_t and its density at the
 *               draft's x_{t-1} (Eq. 2).  In all modes x_0 is the draft's token (Eq. 4).
 *   summary     [R, 5D+1] device, layout as in csd_denoise_lockstep; the last column is
 *               log p(x_T^p) - log q(x_T^q) + sum_{t=2..T} [log p(x^p_{t-1}|x^p_t) -
 *               log q(x^q_{t-1}|x^q_t)] (x^p = x^q in the single-path mode), so csd_verify
 *               applies to it unchanged and gives that ratio's acceptance.
 *   dist2       [R] device float, written: || x^q_0 - x^p_0 ||^2 with the target's own
 *               final sample x^p_0 = mu^p_1 + tau sigma^p_1 eps^p_1.
 *   workspace   csd_ablation_workspace_bytes(draft, target, R, ratio_mode) bytes, 256-byte
 *               aligned; the single-path mode stores the draft's path there
 *               ((T+1) R D floats).
 * The single-path mode runs the draft's rows to the end before the target's.
 */
size_t csd_ablation_workspace_bytes(const csd_head_t* draft, const csd_head_t* target, int64_t n_rows,
                                    int32_t ratio_mode);
int csd_denoise_ablation(const csd_head_t* draft, const csd_head_t* target,
                         const float* z_q, const float* z_p, int64_t n_groups, int32_t gamma,
                         uint64_t seed, uint64_t row_offset, float temperature, int32_t ratio_mode,
                         float* summary, float* dist2, void* workspace, size_t workspace_bytes,
                         void* hip_stream);

/*
 * Split-phase form of the same computation, the way an autoregressive loop runs
 * Alg. 1: the draft head is called once per position as the draft AR model
 * advances ("for i = 1..gamma: x_i ~ q_i"), then the target head once on all
 * positions ("compute p_1..p_gamma in parallel"); the target regenerates the
 * draft's eps_t from the counters (Sec. 3.2), nothing but the summary is kept
 * between the calls.
 *
 * csd_denoise_draft: position (0-based) `position` of every group.  z_q: device
 * [G, C] (one conditioning vector per group).  Fills, in rows g*gamma+position
 * of `summary` (device [G*gamma, 5D+1], the other rows and columns untouched):
 * mu^q_1, log sigma^2_{q,1}, the draft token x_0 (columns [4D,5D): what the
 * draft AR model consumes next) and, in the last column, the draft's half of
 * log Sigma.  Noise counters are the lockstep call's: global row
 * row_offset + g*gamma + position.  Workspace: csd_workspace_bytes(draft,NULL,G).
 *
 * csd_denoise_target: all R = G*gamma rows.  z_p: device [R, C].  Fills mu^p_1,
 * log sigma^2_{p,1} and turns the last column into log Sigma (Eq. 6).  `draft`
 * is consulted for its schedule only.  After both phases the summary holds
 * bit for bit what csd_denoise_lockstep writes.  Workspace:
 * csd_workspace_bytes(NULL,target,R).
 * Errors as csd_denoise_lockstep.
 */
int csd_denoise_draft(const csd_head_t* draft, const float* z_q,
                      int64_t n_groups, int32_t gamma, int32_t position,
                      uint64_t seed, uint64_t row_offset, float temperature,
                      float* summary, void* workspace, size_t workspace_bytes, void* hip_stream);
int csd_denoise_target(const csd_head_t* target, const csd_head_t* draft, const float* z_p,
                       int64_t n_groups, int32_t gamma,
                       uint64_t seed, uint64_t row_offset, float temperature,
                       float* summary, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Plain sampling from one head (target-only mode): x_0 ~ head(.|z) by the same
 * T-step reverse process (Sec. 3.1, Eq. 3), no verification.  Serves pre-filling
 * (Sec. 3.4) and the token from p_{gamma+1} that Alg. 1 returns when all gamma
 * drafts are accepted; for that one pass rng_stream = CSD_STREAM_BONUS and
 * row_offset = the global index of the first group, so its noise is independent
 * of every draft trajectory.  z: device [n_rows, C]; tokens: device [n_rows, D].
 * Workspace: csd_workspace_bytes(head,NULL,n_rows).
 */
int csd_sample(const csd_head_t* head, const float* z, int64_t n_rows,
               uint64_t seed, uint64_t row_offset, int32_t rng_stream, float temperature,
               float* tokens, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Accept test and first-reject scan (Alg. 1; Eq. 7).  Per row
 *   log_ratio = log Sigma + log N(x_0; mu^p_1, (temperature*sigma_{p,1})^2)
 *                         - log N(x_0; mu^q_1, (temperature*sigma_{q,1})^2),
 * r ~ U(0,1) from stream CSD_STREAM_ACCEPT_U; the row is accepted iff
 * log r <= log_ratio (a NaN ratio rejects).  n_accept[g] = number of leading
 * accepted rows of group g (gamma if none is rejected).
 * summary: device [R,5D+1]; n_accept: device int32 [G]; log_ratio (device fp32
 * [R]) and mask (device uint8 [R], 1 = accepted) may be NULL.  gamma <= 64.
 */
int csd_verify(const float* summary, int64_t n_groups, int32_t gamma, int32_t token_dim,
               uint64_t seed, uint64_t row_offset, float temperature,
               int32_t* n_accept, float* log_ratio, uint8_t* mask, void* hip_stream);

/*
 * Acceptance-rejection resampling from max(0,p-q)/Z and emit (Sec. 3.3, Cor. 1;
 * Alg. 1 repeat-until and return).  For each group with n = n_accept[g] < gamma,
 * at its first rejected row j: for k = 0,1,.. propose
 *   x' = mu^p_1 + temperature*sigma_{p,1}*eps'_k,
 *   a = log q(x'|x_1^q) - log Sigma - log p(x'|x_1^p),  alpha_s = max(0, 1-exp(a)),
 * and stop at the first k with u_k <= alpha_s (u_k from CSD_STREAM_RESAMPLE_U).
 * tokens: device fp32 [G, gamma+1, D] = [x_1..x_n, x', 0..]; n_out[g] = n+1, or
 * gamma when the whole group was accepted; trips[g] = trials used (0 if none);
 * flags[g]: CSD_FLAG_* bits.  1 <= max_trips <= 65535.  trips/flags may be NULL.
 */
int csd_resample(const float* summary, const int32_t* n_accept,
                 int64_t n_groups, int32_t gamma, int32_t token_dim,
                 uint64_t seed, uint64_t row_offset, float temperature, int32_t max_trips,
                 float* tokens, int32_t* n_out, int32_t* trips, uint32_t* flags,
                 void* hip_stream);

/*
 * Alg. 1, last line: a group whose gamma drafts were all accepted also emits the
 * target's own sample for position gamma+1.  For every g with n_accept[g] ==
 * gamma: tokens[g, gamma, :] = bonus[g, :] and n_out[g] = gamma+1; other groups
 * are untouched.  tokens [G,gamma+1,D], n_out [G], n_accept [G], bonus [G,D]:
 * device; run after csd_resample on the same stream.
 */
int csd_append_bonus(float* tokens, int32_t* n_out, const int32_t* n_accept, const float* bonus,
                     int64_t n_groups, int32_t gamma, int32_t token_dim, void* hip_stream);

/*
 * Mixture-of-Gaussians output heads (the appendix on other forms of the output
 * distribution): the models emit, per row, p(x) = sum_k pi_k N(x; mu_k, Sigma_k) with
 * diagonal Sigma_k instead of running a diffusion head.  With explicit densities the accept
 * test of Alg. 1 is r <= p(x)/q(x), and the modified distribution max(0, p - q)/Z is
 * sampled by acceptance-rejection with proposal p and threshold max(0, p(x') - q(x'))/p(x').
 * A mixture is three device arrays, fp32: pi [R, K] (>= 0, need not sum to 1; a component
 * with pi = 0 is never drawn), mu [R, K, D], logvar [R, K, D].  1 <= K <= 64, D in {4, 8, 16}.
 *
 * csd_gmm_draft_sample: x [R, D] (device, written) = the draft tokens x_i ~ q_i; the
 *   component comes from stream CSD_STREAM_GMM_PICK slot 0 (first k whose running fp32 sum
 *   of pi reaches u * sum pi), the noise from stream CSD_STREAM_TRAJ slot 0.
 * csd_gmm_verify: as csd_verify with log_ratio = log p(x) - log q(x); outputs as there.
 * csd_gmm_resample: as csd_resample; trial k draws its component from stream
 *   CSD_STREAM_GMM_PICK slot 1+k, its noise from CSD_STREAM_RESAMPLE_N slot k and its
 *   uniform from CSD_STREAM_RESAMPLE_U slot k; x is the array of draft tokens that
 *   csd_gmm_verify judged.  tokens [G, gamma+1, D], n_out, trips, flags as in csd_resample.
 * n_rows / n_groups = 0 is a no-op.  Errors: CSD_EINVAL, CSD_EHIP.
 */
int csd_gmm_draft_sample(const float* pi_q, const float* mu_q, const float* logvar_q, int64_t n_rows,
                         int32_t n_components, int32_t token_dim, uint64_t seed, uint64_t row_offset,
                         float* x, void* hip_stream);
int csd_gmm_verify(const float* x, const float* pi_p, const float* mu_p, const float* logvar_p,
                   const float* pi_q, const float* mu_q, const float* logvar_q, int64_t n_groups,
                   int32_t gamma, int32_t n_components, int32_t token_dim, uint64_t seed,
                   uint64_t row_offset, int32_t* n_accept, float* log_ratio, uint8_t* accept_mask,
                   void* hip_stream);
int csd_gmm_resample(const float* x, const int32_t* n_accept, const float* pi_p, const float* mu_p,
                     const float* logvar_p, const float* pi_q, const float* mu_q, const float* logvar_q,
                     int64_t n_groups, int32_t gamma, int32_t n_components, int32_t token_dim,
                     uint64_t seed, uint64_t row_offset, int32_t max_trips, float* tokens,
                     int32_t* n_out, int32_t* trips, uint32_t* flags, void* hip_stream);


/*
 * Stage-wise access for tests and profiling: one head evaluation
 * (eps_hat, v) = Head(x_t, t, z) for n_rows rows (definition above).
 * x: device [n_rows, D] fp32; z: device [n_rows, C] fp32; t in 1..T;
 * out: device [n_rows, 2D] fp32 = [eps_hat | v].  Workspace as for
 * csd_denoise_lockstep with this head alone.
 */
int csd_head_eval(const csd_head_t* head, const float* x, const float* z, int32_t t,
                  int64_t n_rows, float* out, void* workspace, size_t workspace_bytes,
                  void* hip_stream);

/*
 * Stage-wise access to the generator: out[r, 0:n_cols] (device fp32) for global
 * rows row_offset + r, r < n_rows.  csd_rng_normals: n_cols standard normals
 * (a multiple of 4), element 4b+j from counter block b.  csd_rng_uniforms:
 * n_cols = 1, the 23-bit uniform of block 0.  slot < 65536, stream_id < 65536.
 */
int csd_rng_normals(uint64_t seed, uint64_t row_offset, int64_t n_rows, int32_t slot,
                    int32_t stream_id, int32_t n_cols, float* out, void* hip_stream);
int csd_rng_uniforms(uint64_t seed, uint64_t row_offset, int64_t n_rows, int32_t slot,
                     int32_t stream_id, float* out, void* hip_stream);

/*
 * Stage-wise access to the bf16 MFMA GEMM of the head's dense layers:
 *   C[M,N] = epilogue(A[M,K] * B[N,K]^T + bias[N]),  fp32 accumulation.
 * A, B: device bf16 (raw uint16 bit patterns), dense row-major; bias: device fp32.
 * epilogue 0: identity; 1: SiLU; 2: C(fp32) += gate * (.) with gate device bf16 [M,N].
 * out_f32 != 0 stores C as fp32, else as bf16 (epilogue 2 always fp32).
 * K and N must be multiples of 64; all pointers 16-byte aligned.
 */
int csd_gemm_bf16(const void* A, const void* B, const float* bias, int64_t M, int32_t N, int32_t K,
                  int32_t epilogue, int32_t out_f32, void* C, const void* gate, void* hip_stream);

/*
 * Timing of the dominant kernel (the modulation GEMM of the denoising calls).
 * While enabled, every launch of that kernel is bracketed by two hipEvents on its
 * launch stream (up to `max_launches`; later launches run untimed), and the bf16
 * kernel records the times its first workgroup starts and its last one ends.
 * csd_profile_read waits for the recorded events and returns the sum of the
 * event-to-event durations in milliseconds, the number of launches timed, the
 * sum of their algorithmic flops (2*M*N*K each) and, if ms_sum_on_device is not
 * NULL, the sum of the first-start-to-last-end spans (0 if not available: fp32
 * kernels); it then clears the record.  When several chains share the chip both
 * figures include the time the kernel's workgroups share the compute units with
 * the other chains' kernels (measured: the two agree within a few percent).
 * csd_profile_enable(0) stops recording and frees the events.
 */
int csd_profile_enable(int32_t max_launches);
int csd_profile_read(double* ms_sum, int64_t* launches, double* flops_sum, double* ms_sum_on_device);

/* Message of the last failing call on this thread ("" if none). */
const char* csd_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CSD_H */
