// Internal declarations shared by the translation units of libcsd (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <vector>

#include "../../include/csd.h"

namespace csd {

typedef uint16_t bf16_t;   // storage only; conversions below

__host__ __device__ inline float bf16_to_f32(bf16_t v) {
    union { uint32_t u; float f; } c; c.u = (uint32_t)v << 16; return c.f;
}
// round to nearest even; on the device this is the hardware conversion of gfx950
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__host__ __device__ inline uint32_t pack_bf16x2(float lo, float hi) {
#if defined(__HIP_DEVICE_COMPILE__)
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));   // v_cvt_pk_bf16_f32
#else
    union { uint32_t u; float f; } a, b; a.f = lo; b.f = hi;
    const uint32_t ra = (a.u + 0x7FFFu + ((a.u >> 16) & 1u)) >> 16, rb = (b.u + 0x7FFFu + ((b.u >> 16) & 1u)) >> 16;
    return (ra & 0xFFFFu) | (rb << 16);
#endif
}
__host__ __device__ inline bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xFFFFu); }

// per-step constants of one head's sampler, fp32 copies of host doubles
struct StepCoef {
    float cx;      // coefficient of x_t in mu_t, skip folded in: (1 - gain*beta_t)/sqrt(alpha_t)
    float co;      // coefficient of -o[0:D] in mu_t: beta_t / (sqrt(1-abar_t) sqrt(alpha_t))
    float lmid;    // (log beta_t + log beta~_t)/2: log sigma^2 at v = 0
    float lhalf;   // (log beta_t - log beta~_t)/2: d log sigma^2 / d v
};

// one linear layer on the device: fp32 master copy and, in bf16 mode, a bf16 copy
struct Linear {
    const float* w = nullptr;     // [n_out, n_in]
    const float* b = nullptr;     // [n_out]
    const bf16_t* w16 = nullptr;  // [n_out, n_in] (bf16 mode, large layers only)
    int n_out = 0, n_in = 0;
};

}  // namespace csd

struct csd_head {
    csd_head_cfg_t cfg;
    int device;
    int D, C, W, L, T;
    float ln_eps;
    int reps = 1;                        // head rows per trajectory row: 2 with classifier-free guidance
    float cfg_scale = 0.f;               // guidance scale (reps == 2)
    csd::Linear t1, t2, cond, in, fmod, out;
    csd::Linear out_pad;                 // output layer padded to 64 rows; bf16 copy is [w | w] (2W per row)
    int out_splits = 1;                  // K ranges of the output projection (a fixed property of the head, so that
                                         // every call shape adds the same partial sums in the same order)
    float* d_out_pad = nullptr;          // storage of out_pad (fp32 w, b)
    float* d_in_t = nullptr;             // input projection transposed to [D, W]
    std::vector<csd::Linear> mod, fc1, fc2;
    csd::Linear mod_all;                 // the L modulation layers stacked: [L*3W, W], one GEMM per step
    void* d_mod_all = nullptr;           // its weights (bf16 or fp32 by gemm dtype) ...
    float* d_mod_all_bias = nullptr;     // ... and bias [L*3W]
    std::vector<csd::StepCoef> coef;     // [T+1], entry 0 unused
    std::vector<float> skip_sqrt;        // [T+1]: eps_skip_gain * sqrt(1 - abar_t)
    double ref_log_sigma;                // sum_{t=2..T} D/2 * lmid_t in double
    float* d_weights = nullptr;          // fp32 blob
    csd::bf16_t* d_weights16 = nullptr;  // bf16 copies of the large matrices
    float* d_time_emb = nullptr;         // [T+1, W]
};

namespace csd {

// activation storage type by gemm dtype
enum { ACT_F32 = 0, ACT_BF16 = 1 };

// Epilogues of the GEMM C = A * B^T (+ bias)
enum { EPI_BIAS = 0,        // C = acc + bias
       EPI_BIAS_SILU = 1,   // C = silu(acc + bias)
       EPI_GATE_RES = 2 };  // C(fp32) += gate * (acc + bias)   (stage-wise hook only)

struct GemmArgs {
    const void* A; int lda;        // [M,K] activations (fp32 or bf16)
    const void* B;                 // [N,K] weights, same type as A
    const float* bias;             // [N] fp32
    void* C; int ldc;              // [M,N]; fp32 for EPI_GATE_RES, else activation type
    const void* gate; int ldg;     // [M,N] activation type (EPI_GATE_RES)
    int M, N, K;
    int epi;
    int c_is_f32;                  // output type override: 1 = fp32 even in bf16 mode
    int k_splits;                  // bf16 kernels: > 1 cuts K into that many equal ranges (K % (64 k_splits) == 0); range
    int64_t c_split_stride;        // s writes its partial product to C + s * c_split_stride elements, the bias goes
                                   // into range 0 only; the consumer adds the partials.  0 or 1: off
    unsigned long long* ts;        // optional, device: ts[0] = min start, ts[1] = max end of the workgroups (100 MHz
                                   // constant clock), for profiling; bf16 kernels only
};

hipError_t launch_gemm_f32(const GemmArgs& g, hipStream_t st);
hipError_t launch_gemm_bf16(const GemmArgs& g, hipStream_t st);

// s[k] = silu(E_{t-k} + e) for k = 0 .. n_steps-1 (a batch of consecutive denoising steps); time_emb_t = row t of the table
hipError_t launch_cond_silu(const float* e, const float* time_emb_t, int n_steps, void* s, int act, int64_t R, int W,
                            hipStream_t st);
// start of a block: residual of the previous block (or the input projection), LN, modulation
struct BlockPreArgs {
    int mode;                  // 0 first block, 1 middle, 2 after the last block (see elementwise.hip)
    int act;                   // ACT_F32 | ACT_BF16: type of y, gate, mod (modes 0,1) and u
    float* h;                  // [R,W] fp32 residual stream, read (modes 1,2) and written
    const void* y;             // [R,W] output of the previous block's second linear layer
    const void* gate; int ldg; // [R,ldg] gate of the previous block
    const void* mod; int ldm;  // shift at columns [0,W), scale at [W,2W); fp32 in mode 2
    void* u;                   // [R,W] (mode 2 with bf16: [R,2W] = [hi | lo])
    const float* x; const float* w_in; const float* b_in;   // mode 0: x [R,D], W_in [W,D], b_in [W]
    const float* w_in_t;       // mode 0, optional: W_in transposed to [D,W] (enables the 4-rows-per-wave path)
    float ln_eps; int64_t R; int W; int D;
    int x_div;                 // mode 0: head row i reads x row i / x_div (2 with guidance: cond and uncond rows share x)
};
hipError_t launch_block_pre(const BlockPreArgs& a, hipStream_t st);

struct TransArgs {
    const float* o; int ldo;   // [R, ldo] fp32 output projection: columns [0,D) eps part, [D,2D) v
    int o_splits; int64_t o_split_stride;   // o is the sum of o_splits partial products, o_split_stride floats apart
    int64_t R; int D;
    float* x;                  // [R,D] in: x_t, out: x_{t-1} (not written at t = 1)
    float* acc;                // [R] running 1/2 sum_d (log sigma^2 - lmid_t), t >= 2
    StepCoef coef; int t;
    uint64_t seed, row_offset; float tau;
    int64_t row_stride, row_shift;   // row r of this launch is row r*row_stride + row_shift of the call's summary,
                                     // and global row row_offset + that of the noise counters
    int rng_stream;                  // CSD_STREAM_TRAJ, or CSD_STREAM_BONUS for the target-only bonus sample
    float* summary; int is_target;   // t == 1: writes this head's part of the summary row
    float* tokens;                   // optional [R,D]: t == 1 writes x_0 there instead (plain sampling)
    float* raw_out;            // optional [R,2D]: (eps_hat, v) for csd_head_eval; skips the transition
    float skip_coef;           // eps_skip_gain * sqrt(1 - abar_t), for raw_out only
    int reps; float cfg_scale; // reps == 2: row r's outputs are o[2r] (conditional) and o[2r+1] (unconditional);
                               // eps part = o_u + cfg_scale (o_c - o_u), v part = the conditional one
    // Path-ratio comparison (Table 1).  PATH_PLAIN: acc takes the log-variance part only (under aligned
    // noise the exponents of the two heads' densities cancel, Eq. 6).  PATH_OWN: acc also takes
    // 1/2 ||eps_t||^2, the exponent of this head's density at its own sample.  PATH_FOLLOW: the head does
    // not sample; x_{t-1} is read from path_in and acc takes 1/2 ||(x_{t-1} - mu)/(tau sigma)||^2 (Eq. 2).
    int path_mode;
    const float* path_in;      // [R,D] x_{t-1} of the path to follow (PATH_FOLLOW, t >= 2)
    float* path_out;           // optional [R,D]: x_{t-1} is also stored here (t >= 2)
    float* x0_own;             // optional [R,D]: at t = 1 the head's own sample mu_1 + tau sigma_1 eps_1
};
enum { PATH_PLAIN = 0, PATH_OWN = 1, PATH_FOLLOW = 2 };
hipError_t launch_transition(const TransArgs& a, hipStream_t st);

// x = eps_T from the counters (or a copy of x_src), acc = 0 (or 1/2 ||x_T||^2 if acc_norm), x_store (optional) = x
hipError_t launch_init_x(float* x, float* acc, int64_t R, int D, int T, uint64_t seed, uint64_t row_offset,
                         int64_t row_stride, int64_t row_shift, int rng_stream, int acc_norm, const float* x_src,
                         float* x_store, hipStream_t st);
// dist2[r] = || x_0 of summary row r - x0_own[r] ||^2
hipError_t launch_token_distance(const float* summary, const float* x0_own, float* dist2, int64_t R, int D,
                                 hipStream_t st);
// mode 0: lockstep (acc_q - acc_p + ref); 1: draft phase parks acc_q; 2: target phase finishes from the parked value
hipError_t launch_finish_summary(float* summary, const float* accq, const float* accp, float ref_diff,
                                 int64_t R, int D, int mode, int64_t row_stride, int64_t row_shift, hipStream_t st);
hipError_t launch_append_bonus(float* tokens, int32_t* n_out, const int32_t* n_accept, const float* bonus,
                               int64_t G, int gamma, int D, hipStream_t st);

hipError_t launch_verify(const float* summary, int64_t G, int gamma, int D, uint64_t seed, uint64_t row_offset,
                         float tau, int32_t* n_accept, float* log_ratio, uint8_t* mask, hipStream_t st);
hipError_t launch_resample(const float* summary, const int32_t* n_accept, int64_t G, int gamma, int D,
                           uint64_t seed, uint64_t row_offset, float tau, int max_trips,
                           float* tokens, int32_t* n_out, int32_t* trips, uint32_t* flags, hipStream_t st);
// mixture-of-Gaussians heads (gmm.hip): pi [R,K], mu / logvar [R,K,D]
hipError_t launch_gmm_draft_sample(const float* pi, const float* mu, const float* lv, int64_t R, int K, int D,
                                   uint64_t seed, uint64_t row_offset, float* x, hipStream_t st);
hipError_t launch_gmm_verify(const float* x, const float* pi_p, const float* mu_p, const float* lv_p, const float* pi_q,
                             const float* mu_q, const float* lv_q, int64_t G, int gamma, int K, int D, uint64_t seed,
                             uint64_t row_offset, int32_t* n_accept, float* log_ratio, uint8_t* mask, hipStream_t st);
hipError_t launch_gmm_resample(const float* x, const int32_t* n_accept, const float* pi_p, const float* mu_p,
                               const float* lv_p, const float* pi_q, const float* mu_q, const float* lv_q, int64_t G,
                               int gamma, int K, int D, uint64_t seed, uint64_t row_offset, int max_trips, float* tokens,
                               int32_t* n_out, int32_t* trips, uint32_t* flags, hipStream_t st);
hipError_t launch_rng_normals(uint64_t seed, uint64_t row_offset, int64_t R, int slot, int stream_id, int n_cols,
                              float* out, hipStream_t st);
hipError_t launch_rng_uniforms(uint64_t seed, uint64_t row_offset, int64_t R, int slot, int stream_id,
                               float* out, hipStream_t st);
hipError_t launch_f32_to_bf16(const float* src, bf16_t* dst, size_t n, hipStream_t st);
// dst[r*ld_dst + c] = bf16(src[r*cols + c])
hipError_t launch_f32_to_bf16_rows(const float* src, bf16_t* dst, int rows, int cols, int ld_dst, hipStream_t st);

}  // namespace csd
