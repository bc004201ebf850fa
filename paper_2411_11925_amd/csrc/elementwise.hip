// Row-wise kernels of the head and the sampler: conditioning SiLU, input
// projection, layer-norm + modulation, and the transition kernel that ends a
// denoising step (Gaussian transition of Eq. 3 with the shared noise eps_t,
// log Sigma accumulation of Eq. 6, summary row at t = 1).
#include "internal.hpp"
#include "rng.hpp"

namespace csd {

template <typename T> __device__ __forceinline__ float act_load(const T* p, size_t i);
template <> __device__ __forceinline__ float act_load<float>(const float* p, size_t i) { return p[i]; }
template <> __device__ __forceinline__ float act_load<bf16_t>(const bf16_t* p, size_t i) { return bf16_to_f32(p[i]); }
template <typename T> __device__ __forceinline__ void act_store(T* p, size_t i, float v);
template <> __device__ __forceinline__ void act_store<float>(float* p, size_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void act_store<bf16_t>(bf16_t* p, size_t i, float v) { p[i] = f32_to_bf16(v); }

__device__ __forceinline__ float silu_f(float a) { return a / (1.0f + __expf(-a)); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// ---------------------------------------------------------------- s = silu(E_t + e)
template <typename TAct>
__global__ void k_cond_silu(const float* __restrict__ e, const float* __restrict__ temb, TAct* __restrict__ s,
                            size_t n, int W) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        const int w = (int)(i % (size_t)W);
        act_store<TAct>(s, i, silu_f(e[i] + temb[w]));
    }
}

hipError_t launch_cond_silu(const float* e, const float* temb, void* s, int act, int64_t R, int W, hipStream_t st) {
    const size_t n = (size_t)R * W;
    if (n == 0) return hipSuccess;
    const int threads = 256;
    const size_t want = (n + threads - 1) / threads;
    const int blocks = (int)(want < 16384 ? want : 16384);
    if (act == ACT_BF16) hipLaunchKernelGGL(k_cond_silu<bf16_t>, dim3(blocks), dim3(threads), 0, st, e, temb, (bf16_t*)s, n, W);
    else hipLaunchKernelGGL(k_cond_silu<float>, dim3(blocks), dim3(threads), 0, st, e, temb, (float*)s, n, W);
    return hipGetLastError();
}

// ---------------------------------------------------------------- h = W_in x + b_in
// one thread per (row, output feature); D <= 16 inputs
template <int D>
__global__ void k_inproj(const float* __restrict__ x, const float* __restrict__ w, const float* __restrict__ b,
                         float* __restrict__ h, int64_t R, int W) {
    const int64_t r = blockIdx.y;
    const int o = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= R || o >= W) return;
    float acc = b[o];
#pragma unroll
    for (int d = 0; d < D; ++d) acc = fmaf(w[(size_t)o * D + d], x[r * D + d], acc);
    h[r * W + o] = acc;
}

hipError_t launch_inproj(const float* x, const float* w, const float* b, float* h, int64_t R, int D, int W, hipStream_t st) {
    if (R == 0) return hipSuccess;
    // gridDim.y is limited to 65535: walk the rows in slabs
    for (int64_t r0 = 0; r0 < R; r0 += 65535) {
        const int64_t n = (R - r0 < 65535) ? R - r0 : 65535;
        dim3 grid((W + 255) / 256, (unsigned)n), block(256);
        const float* xs = x + r0 * D; float* hs = h + r0 * W;
        switch (D) {
            case 4: hipLaunchKernelGGL(k_inproj<4>, grid, block, 0, st, xs, w, b, hs, n, W); break;
            case 8: hipLaunchKernelGGL(k_inproj<8>, grid, block, 0, st, xs, w, b, hs, n, W); break;
            case 16: hipLaunchKernelGGL(k_inproj<16>, grid, block, 0, st, xs, w, b, hs, n, W); break;
            default: return hipErrorInvalidValue;
        }
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------- LN statistics of one row by one wave
__device__ __forceinline__ void row_stats(const float* __restrict__ hrow, int W, int lane, float ln_eps,
                                          float& mean, float& rstd) {
    float s = 0.f;
    for (int j = lane; j < W; j += 64) s += hrow[j];
    mean = wave_sum(s) / (float)W;
    float q = 0.f;
    for (int j = lane; j < W; j += 64) { const float d = hrow[j] - mean; q = fmaf(d, d, q); }
    rstd = 1.0f / sqrtf(wave_sum(q) / (float)W + ln_eps);
}

// ---------------------------------------------------------------- u = LN(h)*(1+scale)+shift
// OUT_SPLIT writes u as two bf16 halves [hi | lo] (lo = bf16(u - hi)) into a row of
// 2W values, so that a bf16 GEMM against [w | w] sees u to ~2^-17 relative.
enum { OUT_SAME = 0, OUT_SPLIT = 1 };
template <typename TMod, typename TOut, int MODE>
__global__ void k_ln_mod(const float* __restrict__ h, const TMod* __restrict__ mod, int ldm, TOut* __restrict__ u,
                         float ln_eps, int64_t R, int W) {
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (r >= R) return;
    const float* hrow = h + r * W;
    float mean, rstd;
    row_stats(hrow, W, lane, ln_eps, mean, rstd);
    const TMod* m = mod + r * (size_t)ldm;
    for (int j = lane; j < W; j += 64) {
        const float v = (hrow[j] - mean) * rstd;
        const float uv = fmaf(v, 1.0f + act_load<TMod>(m, W + j), act_load<TMod>(m, j));
        if (MODE == OUT_SPLIT) {
            const bf16_t hi = f32_to_bf16(uv);
            ((bf16_t*)u)[(size_t)r * 2 * W + j] = hi;
            ((bf16_t*)u)[(size_t)r * 2 * W + W + j] = f32_to_bf16(uv - bf16_to_f32(hi));
        } else {
            act_store<TOut>(u, (size_t)r * W + j, uv);
        }
    }
}

hipError_t launch_ln_mod(const float* h, const void* mod, int ldm, int mod_is_f32, void* u, int out_mode,
                         float ln_eps, int64_t R, int W, hipStream_t st) {
    if (R == 0) return hipSuccess;
    const int rows_per_block = 4;
    dim3 grid((unsigned)((R + rows_per_block - 1) / rows_per_block)), block(64 * rows_per_block);
    if (out_mode == LN_OUT_F32 && mod_is_f32)
        hipLaunchKernelGGL((k_ln_mod<float, float, OUT_SAME>), grid, block, 0, st, h, (const float*)mod, ldm, (float*)u, ln_eps, R, W);
    else if (out_mode == LN_OUT_BF16 && !mod_is_f32)
        hipLaunchKernelGGL((k_ln_mod<bf16_t, bf16_t, OUT_SAME>), grid, block, 0, st, h, (const bf16_t*)mod, ldm, (bf16_t*)u, ln_eps, R, W);
    else if (out_mode == LN_OUT_BF16_SPLIT && mod_is_f32)
        hipLaunchKernelGGL((k_ln_mod<float, bf16_t, OUT_SPLIT>), grid, block, 0, st, h, (const float*)mod, ldm, (bf16_t*)u, ln_eps, R, W);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

// ---------------------------------------------------------------- end of a denoising step
// o = (eps_hat part, v part) of the output projection, [R, ldo] fp32.  The D lanes of a
// row take the reverse transition of Eq. 3 with eps_t regenerated from the counter RNG.
template <int D>
__global__ void k_transition(TransArgs a) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t r = i / D;
    const int d = (int)(i % D);
    if (r >= a.R) return;                      // whole D-lane segments drop out together
    const float o_eps = a.o[r * a.ldo + d], o_v = a.o[r * a.ldo + D + d];
    const float x = a.x[r * D + d];
    if (a.raw_out) {
        a.raw_out[r * 2 * D + d] = fmaf(a.skip_coef, x, o_eps);
        a.raw_out[r * 2 * D + D + d] = o_v;
        return;
    }
    float nrm[4];
    normals4(a.seed, a.row_offset + (uint64_t)r, (uint32_t)(a.t - 1), CSD_STREAM_TRAJ, (uint32_t)(d >> 2), nrm);
    const float eps = nrm[d & 3];
    const float lv = fmaf(o_v, a.coef.lhalf, a.coef.lmid);
    const float mu = fmaf(a.coef.cx, x, -a.coef.co * o_eps);
    const float xn = fmaf(a.tau * expf(0.5f * lv), eps, mu);
    if (a.t >= 2) {
        a.x[r * D + d] = xn;
        float vs = o_v;                       // sum_d v_d over the D lanes of the row
#pragma unroll
        for (int o = D / 2; o >= 1; o >>= 1) vs += __shfl_xor(vs, o, 64);
        if (d == 0) a.acc[r] += 0.5f * a.coef.lhalf * vs;
    } else {
        float* srow = a.summary + r * (5 * D + 1);
        if (a.is_target) {
            srow[d] = mu; srow[D + d] = lv;
        } else {
            srow[2 * D + d] = mu; srow[3 * D + d] = lv; srow[4 * D + d] = xn;
        }
    }
}

hipError_t launch_transition(const TransArgs& a, hipStream_t st) {
    if (a.R == 0) return hipSuccess;
    const int64_t n = a.R * a.D;
    dim3 grid((unsigned)((n + 255) / 256)), block(256);
    switch (a.D) {
        case 4: hipLaunchKernelGGL(k_transition<4>, grid, block, 0, st, a); break;
        case 8: hipLaunchKernelGGL(k_transition<8>, grid, block, 0, st, a); break;
        case 16: hipLaunchKernelGGL(k_transition<16>, grid, block, 0, st, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------- x_T = eps_T for both models
__global__ void k_init_x(float* __restrict__ xq, float* __restrict__ xp, float* __restrict__ accq,
                         float* __restrict__ accp, int64_t R, int D, int T, uint64_t seed, uint64_t row_offset) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // one thread per (row, block of 4)
    const int nb = D >> 2;
    if (i >= R * nb) return;
    const int64_t r = i / nb; const int b = (int)(i % nb);
    float n[4];
    normals4(seed, row_offset + (uint64_t)r, (uint32_t)T, CSD_STREAM_TRAJ, (uint32_t)b, n);
#pragma unroll
    for (int j = 0; j < 4; ++j) { xq[r * D + 4 * b + j] = n[j]; xp[r * D + 4 * b + j] = n[j]; }
    if (b == 0) { accq[r] = 0.f; accp[r] = 0.f; }
}

hipError_t launch_init_x(float* xq, float* xp, float* accq, float* accp, int64_t R, int D, int T,
                         uint64_t seed, uint64_t row_offset, hipStream_t st) {
    const int64_t n = R * (D >> 2);
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_init_x, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, xq, xp, accq, accp, R, D, T, seed, row_offset);
    return hipGetLastError();
}

// log Sigma = (acc_q - acc_p) + (schedule reference difference, 0 for equal schedules)
__global__ void k_finish_summary(float* __restrict__ summary, const float* __restrict__ accq,
                                 const float* __restrict__ accp, float ref_diff, int64_t R, int D) {
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r < R) summary[r * (5 * D + 1) + 5 * D] = (accq[r] - accp[r]) + ref_diff;
}

hipError_t launch_finish_summary(float* summary, const float* accq, const float* accp, float ref_diff,
                                 int64_t R, int D, hipStream_t st) {
    if (R == 0) return hipSuccess;
    hipLaunchKernelGGL(k_finish_summary, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, st, summary, accq, accp, ref_diff, R, D);
    return hipGetLastError();
}

// ---------------------------------------------------------------- generator access for tests
__global__ void k_rng_normals(uint64_t seed, uint64_t row_offset, int64_t R, int slot, int stream_id, int n_cols,
                              float* __restrict__ out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int nb = n_cols >> 2;
    if (i >= R * nb) return;
    const int64_t r = i / nb; const int b = (int)(i % nb);
    float n[4];
    normals4(seed, row_offset + (uint64_t)r, (uint32_t)slot, (uint32_t)stream_id, (uint32_t)b, n);
#pragma unroll
    for (int j = 0; j < 4; ++j) out[r * n_cols + 4 * b + j] = n[j];
}

__global__ void k_rng_uniforms(uint64_t seed, uint64_t row_offset, int64_t R, int slot, int stream_id,
                               float* __restrict__ out) {
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r < R) out[r] = uniform_at(seed, row_offset + (uint64_t)r, (uint32_t)slot, (uint32_t)stream_id);
}

hipError_t launch_rng_normals(uint64_t seed, uint64_t row_offset, int64_t R, int slot, int stream_id, int n_cols,
                              float* out, hipStream_t st) {
    const int64_t n = R * (n_cols >> 2);
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_rng_normals, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, seed, row_offset, R, slot, stream_id, n_cols, out);
    return hipGetLastError();
}

hipError_t launch_rng_uniforms(uint64_t seed, uint64_t row_offset, int64_t R, int slot, int stream_id,
                               float* out, hipStream_t st) {
    if (R == 0) return hipSuccess;
    hipLaunchKernelGGL(k_rng_uniforms, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, st, seed, row_offset, R, slot, stream_id, out);
    return hipGetLastError();
}

__global__ void k_f32_to_bf16(const float* __restrict__ src, bf16_t* __restrict__ dst, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = f32_to_bf16(src[i]);
}

hipError_t launch_f32_to_bf16(const float* src, bf16_t* dst, size_t n, hipStream_t st) {
    if (n == 0) return hipSuccess;
    const size_t want = (n + 255) / 256;
    hipLaunchKernelGGL(k_f32_to_bf16, dim3((unsigned)(want < 8192 ? want : 8192)), dim3(256), 0, st, src, dst, n);
    return hipGetLastError();
}

__global__ void k_f32_to_bf16_rows(const float* __restrict__ src, bf16_t* __restrict__ dst, int rows, int cols, int ld_dst) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows * cols) dst[(size_t)(i / cols) * ld_dst + i % cols] = f32_to_bf16(src[i]);
}

hipError_t launch_f32_to_bf16_rows(const float* src, bf16_t* dst, int rows, int cols, int ld_dst, hipStream_t st) {
    const int n = rows * cols;
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_f32_to_bf16_rows, dim3((n + 255) / 256), dim3(256), 0, st, src, dst, rows, cols, ld_dst);
    return hipGetLastError();
}

}  // namespace csd
