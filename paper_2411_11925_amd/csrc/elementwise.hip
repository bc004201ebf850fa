// Row-wise kernels of the head and the sampler: conditioning SiLU, the fused start of a
// block (input projection or residual, layer-norm, modulation), and the transition kernel
// that ends a denoising step (Gaussian transition of Eq. 3 with the shared noise eps_t,
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
                            size_t n_one, int n_steps, int W) {
    // s[k, r, :] = silu(e[r, :] + E[t_first - k, :]) for the steps k = 0 .. n_steps-1 of a batch;
    // temb points at row t_first of the table, earlier steps are the rows before it
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x, n = n_one * (size_t)n_steps;
    for (; i < n; i += stride) {
        const size_t k = i / n_one, j = i - k * n_one;
        const int w = (int)(j % (size_t)W);
        act_store<TAct>(s, i, silu_f(e[j] + temb[w - (ptrdiff_t)k * W]));
    }
}

// ---------------------------------------------------------------- start of a block
// One wave per row, the row held in registers, one pass over memory:
//   FIRST : h = W_in x + b_in                      (input projection of the head)
//   MIDDLE: h += gate_prev * y_prev                (residual of the previous block)
//   FINAL : same, then the last modulation comes in fp32
// then LN statistics (two-pass, in registers) and u = LN(h)*(1+scale)+shift.
// Writes h (fp32) and u.  With TAct = bf16 the FINAL u is written as a [hi | lo] bf16
// pair (lo = bf16(u - hi)), 2W per row, so that a bf16 GEMM against [w | w] sees u to
// ~2^-17 relative.
enum { PRE_FIRST = 0, PRE_MIDDLE = 1, PRE_FINAL = 2 };

template <typename T> __device__ __forceinline__ void load4(const T* p, float v[4]);
template <> __device__ __forceinline__ void load4<float>(const float* p, float v[4]) {
    const float4 t = *reinterpret_cast<const float4*>(p); v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
template <> __device__ __forceinline__ void load4<bf16_t>(const bf16_t* p, float v[4]) {
    const uint2 t = *reinterpret_cast<const uint2*>(p);
    v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xFFFF0000u);
    v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xFFFF0000u);
}
template <typename T> __device__ __forceinline__ void store4(T* p, const float v[4]);
template <> __device__ __forceinline__ void store4<float>(float* p, const float v[4]) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
}
template <> __device__ __forceinline__ void store4<bf16_t>(bf16_t* p, const float v[4]) {
    *reinterpret_cast<uint2*>(p) = make_uint2(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]));
}

// Vector form (W % 4 == 0): a workgroup takes 8 rows of one step, a thread 4 consecutive
// columns, so the 16 bytes of the time embedding are loaded once for the 8 rows and the index
// arithmetic has no division.  Same operations per element as the scalar kernel.
template <typename TAct>
__global__ __launch_bounds__(256) void k_cond_silu_v4(const float* __restrict__ e, const float* __restrict__ temb,
                                                     TAct* __restrict__ s, int64_t R, int W) {
    constexpr int ROWS = 8;
    const int64_t r0 = (int64_t)blockIdx.x * ROWS;
    const int k = blockIdx.y;
    const float* trow = temb - (ptrdiff_t)k * W;
    TAct* sk = s + (size_t)k * (size_t)R * W;
    for (int c = threadIdx.x * 4; c < W; c += 256 * 4) {
        float t4[4];
        load4<float>(trow + c, t4);
#pragma unroll
        for (int rr = 0; rr < ROWS; ++rr) {
            const int64_t r = r0 + rr;
            if (r >= R) break;
            float e4[4], v[4];
            load4<float>(e + r * W + c, e4);
#pragma unroll
            for (int q = 0; q < 4; ++q) v[q] = silu_f(e4[q] + t4[q]);
            store4<TAct>(sk + r * W + c, v);
        }
    }
}

hipError_t launch_cond_silu(const float* e, const float* temb_first, int n_steps, void* s, int act, int64_t R, int W,
                            hipStream_t st) {
    const size_t n_one = (size_t)R * W, n = n_one * (size_t)n_steps;
    if (n == 0) return hipSuccess;
    if (W % 4 == 0 && n_steps <= 65535 && (((uintptr_t)e | (uintptr_t)temb_first | (uintptr_t)s) & 15u) == 0) {
        dim3 grid((unsigned)((R + 7) / 8), (unsigned)n_steps), block(256);
        if (act == ACT_BF16) hipLaunchKernelGGL(k_cond_silu_v4<bf16_t>, grid, block, 0, st, e, temb_first, (bf16_t*)s, R, W);
        else hipLaunchKernelGGL(k_cond_silu_v4<float>, grid, block, 0, st, e, temb_first, (float*)s, R, W);
        return hipGetLastError();
    }
    const int threads = 256;
    const size_t want = (n + threads - 1) / threads;
    const int blocks = (int)(want < 16384 ? want : 16384);
    if (act == ACT_BF16) hipLaunchKernelGGL(k_cond_silu<bf16_t>, dim3(blocks), dim3(threads), 0, st, e, temb_first, (bf16_t*)s, n_one, n_steps, W);
    else hipLaunchKernelGGL(k_cond_silu<float>, dim3(blocks), dim3(threads), 0, st, e, temb_first, (float*)s, n_one, n_steps, W);
    return hipGetLastError();
}

// NCH = W / 256 chunks of 4 consecutive features per lane (fast path); NCH = 0: any W % 64 == 0,
// one feature per lane and step, three passes (the row is re-read from cache instead of registers).
template <typename TAct, int MODE, int D, int NCH>
__global__ __launch_bounds__(256) void k_block_pre(BlockPreArgs a) {
    const int lane = threadIdx.x & 63;
    const int64_t r = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (r >= a.R) return;
    const int W = a.W;
    float* hrow = a.h + r * W;
    const TAct* yrow = (const TAct*)a.y + r * (size_t)W;
    const TAct* grow = (const TAct*)a.gate + r * (size_t)a.ldg;
    float xr[D];
    if (MODE == PRE_FIRST) {
#pragma unroll
        for (int d = 0; d < D; ++d) xr[d] = a.x[(r / a.x_div) * D + d];
    }
    auto h_at = [&](int j, float out[4], int n) {        // n consecutive features from j
        if (MODE == PRE_FIRST) {
            for (int e = 0; e < n; ++e) {
                float acc = a.b_in[j + e];
#pragma unroll
                for (int d = 0; d < D; ++d) acc = fmaf(a.w_in[(size_t)(j + e) * D + d], xr[d], acc);
                out[e] = acc;
            }
        } else if (n == 4) {
            float hv[4], yv[4], gv[4];
            load4<float>(hrow + j, hv); load4<TAct>(yrow + j, yv); load4<TAct>(grow + j, gv);
#pragma unroll
            for (int e = 0; e < 4; ++e) out[e] = fmaf(gv[e], yv[e], hv[e]);
        } else {
            out[0] = fmaf(act_load<TAct>(grow, j), act_load<TAct>(yrow, j), hrow[j]);
        }
    };
    auto emit = [&](int j, const float hv[4], int n, float mean, float rstd) {
        float sh[4], sc[4], uv[4];
        if (n == 4) {
            if (MODE == PRE_FINAL) { load4<float>((const float*)a.mod + r * (size_t)a.ldm + j, sh); load4<float>((const float*)a.mod + r * (size_t)a.ldm + W + j, sc); }
            else { load4<TAct>((const TAct*)a.mod + r * (size_t)a.ldm + j, sh); load4<TAct>((const TAct*)a.mod + r * (size_t)a.ldm + W + j, sc); }
        } else {
            if (MODE == PRE_FINAL) { sh[0] = ((const float*)a.mod)[r * (size_t)a.ldm + j]; sc[0] = ((const float*)a.mod)[r * (size_t)a.ldm + W + j]; }
            else { sh[0] = act_load<TAct>((const TAct*)a.mod + r * (size_t)a.ldm, j); sc[0] = act_load<TAct>((const TAct*)a.mod + r * (size_t)a.ldm, W + j); }
        }
        for (int e = 0; e < n; ++e) uv[e] = fmaf((hv[e] - mean) * rstd, 1.0f + sc[e], sh[e]);
        if (MODE == PRE_FINAL && sizeof(TAct) == 2) {        // [hi | lo] split
            bf16_t* urow = (bf16_t*)a.u + r * (size_t)2 * W;
            float lo[4];
            for (int e = 0; e < n; ++e) lo[e] = uv[e] - bf16_to_f32(f32_to_bf16(uv[e]));
            if (n == 4) { store4<bf16_t>(urow + j, uv); store4<bf16_t>(urow + W + j, lo); }
            else { urow[j] = f32_to_bf16(uv[0]); urow[W + j] = f32_to_bf16(lo[0]); }
        } else {
            TAct* urow = (TAct*)a.u + r * (size_t)W;
            if (n == 4) store4<TAct>(urow + j, uv); else act_store<TAct>(urow, j, uv[0]);
        }
    };
    if (NCH > 0) {
        float hv[NCH > 0 ? NCH : 1][4];
        float s = 0.f;
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            h_at((c * 64 + lane) * 4, hv[c], 4);
            s += (hv[c][0] + hv[c][1]) + (hv[c][2] + hv[c][3]);
        }
        const float mean = wave_sum(s) / (float)W;
        float q = 0.f;
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e) { const float d = hv[c][e] - mean; q = fmaf(d, d, q); }
        const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)W + a.ln_eps);
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int j = (c * 64 + lane) * 4;
            if (MODE != PRE_FINAL) store4<float>(hrow + j, hv[c]);     // nobody reads h after the last block
            emit(j, hv[c], 4, mean, rstd);
        }
    } else {
        float s = 0.f, v[4];
        for (int j = lane; j < W; j += 64) { h_at(j, v, 1); hrow[j] = v[0]; s += v[0]; }   // pass 1 writes h
        const float mean = wave_sum(s) / (float)W;
        float q = 0.f;
        for (int j = lane; j < W; j += 64) { const float d = hrow[j] - mean; q = fmaf(d, d, q); }
        const float rstd = 1.0f / sqrtf(wave_sum(q) / (float)W + a.ln_eps);
        for (int j = lane; j < W; j += 64) { v[0] = hrow[j]; emit(j, v, 1, mean, rstd); }
    }
}

// First block, fast path: h = W_in x + b_in for FOUR rows per wave, so that each 16-byte
// piece of the (transposed, [D][W]) input weights is loaded once per four rows; then the
// same LN + modulation as above.  The row is streamed in chunks of 256 columns (h is written
// in the first sweep and read back - from L2 - for the centred variance and for u), which
// keeps the kernel at a few dozen registers: it is bandwidth-bound and wants many waves.
template <typename TAct, int D>
__global__ __launch_bounds__(256) void k_block_first(BlockPreArgs a) {
    constexpr int RPW = 4;
    const int lane = threadIdx.x & 63;
    const int64_t r0 = ((int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6)) * RPW;
    if (r0 >= a.R) return;
    const int W = a.W, nch = W / 256;
    const float* __restrict__ w_src = a.w_in;
    float xr[RPW][D];
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) {
        const int64_t r = (r0 + rr < a.R) ? r0 + rr : a.R - 1;
#pragma unroll
        for (int d = 0; d < D; ++d)      // the same value in every lane: keep it in a scalar register
            xr[rr][d] = __uint_as_float(__builtin_amdgcn_readfirstlane(__float_as_uint(a.x[(r / a.x_div) * D + d])));
    }
    float s[RPW], mean[RPW], q[RPW], rstd[RPW];
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) { s[rr] = 0.f; q[rr] = 0.f; }
#pragma unroll 1
    for (int c = 0; c < nch; ++c) {
        const int j = (c * 64 + lane) * 4;
        float hv[RPW][4], b4[4];
        load4<float>(a.b_in + j, b4);
#pragma unroll
        for (int rr = 0; rr < RPW; ++rr)
#pragma unroll
            for (int e = 0; e < 4; ++e) hv[rr][e] = b4[e];
#pragma unroll
        for (int d = 0; d < D; ++d) {
            float w4[4];
            load4<float>(w_src + (size_t)d * W + j, w4);
#pragma unroll
            for (int rr = 0; rr < RPW; ++rr)
#pragma unroll
                for (int e = 0; e < 4; ++e) hv[rr][e] = fmaf(w4[e], xr[rr][d], hv[rr][e]);
        }
#pragma unroll
        for (int rr = 0; rr < RPW; ++rr) {
            s[rr] += (hv[rr][0] + hv[rr][1]) + (hv[rr][2] + hv[rr][3]);
            if (r0 + rr < a.R) store4<float>(a.h + (r0 + rr) * W + j, hv[rr]);
        }
    }
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) mean[rr] = wave_sum(s[rr]) / (float)W;
#pragma unroll 1
    for (int c = 0; c < nch; ++c) {
        const int j = (c * 64 + lane) * 4;
#pragma unroll
        for (int rr = 0; rr < RPW; ++rr) {
            if (r0 + rr >= a.R) continue;
            float hv[4];
            load4<float>(a.h + (r0 + rr) * W + j, hv);
#pragma unroll
            for (int e = 0; e < 4; ++e) { const float d = hv[e] - mean[rr]; q[rr] = fmaf(d, d, q[rr]); }
        }
    }
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr) rstd[rr] = 1.0f / sqrtf(wave_sum(q[rr]) / (float)W + a.ln_eps);
#pragma unroll 1
    for (int c = 0; c < nch; ++c) {
        const int j = (c * 64 + lane) * 4;
#pragma unroll
        for (int rr = 0; rr < RPW; ++rr) {
            const int64_t r = r0 + rr;
            if (r >= a.R) continue;
            const TAct* mrow = (const TAct*)a.mod + r * (size_t)a.ldm;
            float hv[4], sh[4], sc[4], uv[4];
            load4<float>(a.h + r * W + j, hv);
            load4<TAct>(mrow + j, sh); load4<TAct>(mrow + W + j, sc);
#pragma unroll
            for (int e = 0; e < 4; ++e) uv[e] = fmaf((hv[e] - mean[rr]) * rstd[rr], 1.0f + sc[e], sh[e]);
            store4<TAct>((TAct*)a.u + r * (size_t)W + j, uv);
        }
    }
}

template <typename TAct, int D>
static bool launch_block_first(const BlockPreArgs& a, hipStream_t st) {
    if (!a.w_in_t || a.W % 256 != 0 || a.ldm % 4 != 0) return false;
    BlockPreArgs b = a;
    b.w_in = a.w_in_t;
    dim3 grid((unsigned)((a.R + 15) / 16)), block(256);
    hipLaunchKernelGGL((k_block_first<TAct, D>), grid, block, 0, st, b);
    return true;
}

template <typename TAct, int MODE, int D>
static void launch_block_pre_nch(const BlockPreArgs& a, dim3 grid, dim3 block, hipStream_t st) {
    const bool vec = a.W % 256 == 0 && a.ldg % 4 == 0 && a.ldm % 4 == 0;
    switch (vec ? a.W / 256 : 0) {
        case 2: hipLaunchKernelGGL((k_block_pre<TAct, MODE, D, 2>), grid, block, 0, st, a); break;
        case 3: hipLaunchKernelGGL((k_block_pre<TAct, MODE, D, 3>), grid, block, 0, st, a); break;
        case 4: hipLaunchKernelGGL((k_block_pre<TAct, MODE, D, 4>), grid, block, 0, st, a); break;
        case 5: hipLaunchKernelGGL((k_block_pre<TAct, MODE, D, 5>), grid, block, 0, st, a); break;
        case 6: hipLaunchKernelGGL((k_block_pre<TAct, MODE, D, 6>), grid, block, 0, st, a); break;
        case 8: hipLaunchKernelGGL((k_block_pre<TAct, MODE, D, 8>), grid, block, 0, st, a); break;
        default: hipLaunchKernelGGL((k_block_pre<TAct, MODE, D, 0>), grid, block, 0, st, a); break;
    }
}

template <typename TAct, int MODE>
static hipError_t launch_block_pre_d(const BlockPreArgs& a, dim3 grid, dim3 block, hipStream_t st) {
    if (MODE != PRE_FIRST) { launch_block_pre_nch<TAct, MODE, 4>(a, grid, block, st); return hipSuccess; }
    switch (a.D) {
        case 4: if (!launch_block_first<TAct, 4>(a, st)) launch_block_pre_nch<TAct, MODE, 4>(a, grid, block, st); break;
        case 8: if (!launch_block_first<TAct, 8>(a, st)) launch_block_pre_nch<TAct, MODE, 8>(a, grid, block, st); break;
        case 16: if (!launch_block_first<TAct, 16>(a, st)) launch_block_pre_nch<TAct, MODE, 16>(a, grid, block, st); break;
        default: return hipErrorInvalidValue;
    }
    return hipSuccess;
}

hipError_t launch_block_pre(const BlockPreArgs& a, hipStream_t st) {
    if (a.R == 0) return hipSuccess;
    dim3 grid((unsigned)((a.R + 3) / 4)), block(256);
    hipError_t e = hipErrorInvalidValue;
    if (a.act == ACT_BF16) {
        if (a.mode == PRE_FIRST) e = launch_block_pre_d<bf16_t, PRE_FIRST>(a, grid, block, st);
        else if (a.mode == PRE_MIDDLE) e = launch_block_pre_d<bf16_t, PRE_MIDDLE>(a, grid, block, st);
        else if (a.mode == PRE_FINAL) e = launch_block_pre_d<bf16_t, PRE_FINAL>(a, grid, block, st);
    } else {
        if (a.mode == PRE_FIRST) e = launch_block_pre_d<float, PRE_FIRST>(a, grid, block, st);
        else if (a.mode == PRE_MIDDLE) e = launch_block_pre_d<float, PRE_MIDDLE>(a, grid, block, st);
        else if (a.mode == PRE_FINAL) e = launch_block_pre_d<float, PRE_FINAL>(a, grid, block, st);
    }
    return e != hipSuccess ? e : hipGetLastError();
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
    const int64_t ro = r * a.reps;
    // the output projection arrives as o_splits partial products (split-K), added here in order
    float o_eps = a.o[ro * a.ldo + d];
    float o_v = a.o[ro * a.ldo + D + d];
    for (int s = 1; s < a.o_splits; ++s) {
        o_eps += a.o[s * a.o_split_stride + ro * a.ldo + d];
        o_v += a.o[s * a.o_split_stride + ro * a.ldo + D + d];
    }
    if (a.reps == 2) {                         // classifier-free guidance: eps_u + s (eps_c - eps_u)
        float o_u = a.o[(ro + 1) * a.ldo + d];
        for (int s = 1; s < a.o_splits; ++s) o_u += a.o[s * a.o_split_stride + (ro + 1) * a.ldo + d];
        o_eps = fmaf(a.cfg_scale, o_eps - o_u, o_u);
    }
    const float x = a.x[r * D + d];
    if (a.raw_out) {
        a.raw_out[r * 2 * D + d] = fmaf(a.skip_coef, x, o_eps);
        a.raw_out[r * 2 * D + D + d] = o_v;
        return;
    }
    float nrm[4];
    const int64_t sr = r * a.row_stride + a.row_shift;      // row of the call's summary / global row behind row_offset
    normals4(a.seed, a.row_offset + (uint64_t)sr, (uint32_t)(a.t - 1), (uint32_t)a.rng_stream, (uint32_t)(d >> 2), nrm);
    const float eps = nrm[d & 3];
    const float lv = fmaf(o_v, a.coef.lhalf, a.coef.lmid);
    const float mu = fmaf(a.coef.cx, x, -a.coef.co * o_eps);
    const float sd = a.tau * expf(0.5f * lv);
    float xn = fmaf(sd, eps, mu);
    if (a.t >= 2) {
        float vs = o_v;                       // sum_d v_d over the D lanes of the row
#pragma unroll
        for (int o = D / 2; o >= 1; o >>= 1) vs += __shfl_xor(vs, o, 64);
        float add = 0.5f * a.coef.lhalf * vs;
        if (a.path_mode != PATH_PLAIN) {      // the exponent of this step's density (uniform over the launch)
            float q = eps;
            if (a.path_mode == PATH_FOLLOW) { xn = a.path_in[r * D + d]; q = (xn - mu) / sd; }
            q *= q;
#pragma unroll
            for (int o = D / 2; o >= 1; o >>= 1) q += __shfl_xor(q, o, 64);
            add += 0.5f * q;
        }
        a.x[r * D + d] = xn;
        if (a.path_out) a.path_out[r * D + d] = xn;
        if (d == 0) a.acc[r] += add;
    } else if (a.tokens) {
        a.tokens[r * D + d] = xn;             // plain sampling: x_0 itself
    } else {
        float* srow = a.summary + sr * (5 * D + 1);
        if (a.is_target) {
            srow[d] = mu; srow[D + d] = lv;
        } else {
            srow[2 * D + d] = mu; srow[3 * D + d] = lv; srow[4 * D + d] = xn;
        }
        if (a.x0_own) a.x0_own[r * D + d] = xn;
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

// ---------------------------------------------------------------- x_T = eps_T, accumulator = 0
__global__ void k_init_x(float* __restrict__ x, float* __restrict__ acc, int64_t R, int D, int T, uint64_t seed,
                         uint64_t row_offset, int64_t row_stride, int64_t row_shift, int rng_stream, int acc_norm,
                         const float* __restrict__ x_src, float* __restrict__ x_store) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;   // one thread per (row, block of 4)
    const int nb = D >> 2;
    if (i >= R * nb) return;                   // the nb lanes of a row drop out together
    const int64_t r = i / nb; const int b = (int)(i % nb);
    float n[4];
    if (x_src) {
#pragma unroll
        for (int j = 0; j < 4; ++j) n[j] = x_src[r * D + 4 * b + j];
    } else {
        normals4(seed, row_offset + (uint64_t)(r * row_stride + row_shift), (uint32_t)T, (uint32_t)rng_stream, (uint32_t)b, n);
    }
    float q = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        x[r * D + 4 * b + j] = n[j];
        if (x_store) x_store[r * D + 4 * b + j] = n[j];
        q = fmaf(n[j], n[j], q);
    }
    for (int o = nb / 2; o >= 1; o >>= 1) q += __shfl_xor(q, o, 64);      // nb is 1, 2 or 4
    if (b == 0) acc[r] = acc_norm ? 0.5f * q : 0.f;
}

hipError_t launch_init_x(float* x, float* acc, int64_t R, int D, int T, uint64_t seed, uint64_t row_offset,
                         int64_t row_stride, int64_t row_shift, int rng_stream, int acc_norm, const float* x_src,
                         float* x_store, hipStream_t st) {
    const int64_t n = R * (D >> 2);
    if (n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_init_x, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, x, acc, R, D, T, seed, row_offset,
                       row_stride, row_shift, rng_stream, acc_norm, x_src, x_store);
    return hipGetLastError();
}

// squared distance between the draft token of a summary row and the target's own final sample
__global__ void k_token_distance(const float* __restrict__ summary, const float* __restrict__ x0_own,
                                 float* __restrict__ dist2, int64_t R, int D) {
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= R) return;
    const float* x0 = summary + r * (5 * D + 1) + 4 * D;
    float q = 0.f;
    for (int d = 0; d < D; ++d) { const float df = x0[d] - x0_own[r * D + d]; q = fmaf(df, df, q); }
    dist2[r] = q;
}

hipError_t launch_token_distance(const float* summary, const float* x0_own, float* dist2, int64_t R, int D,
                                 hipStream_t st) {
    if (R == 0) return hipSuccess;
    hipLaunchKernelGGL(k_token_distance, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, st, summary, x0_own, dist2, R, D);
    return hipGetLastError();
}

// The last column of the summary.  mode 0 (lockstep): log Sigma = (acc_q - acc_p) + ref, ref = the
// schedule reference difference (0 for equal schedules).  mode 1 (draft phase): the draft's half,
// acc_q, is parked there.  mode 2 (target phase): log Sigma = (parked - acc_p) + ref - the same
// operations on the same values as mode 0, so both routes give the same bits.
__global__ void k_finish_summary(float* __restrict__ summary, const float* __restrict__ accq,
                                 const float* __restrict__ accp, float ref_diff, int64_t R, int D, int mode,
                                 int64_t row_stride, int64_t row_shift) {
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= R) return;
    float* slot = summary + (r * row_stride + row_shift) * (5 * D + 1) + 5 * D;
    if (mode == 0) *slot = (accq[r] - accp[r]) + ref_diff;
    else if (mode == 1) *slot = accq[r];
    else *slot = (*slot - accp[r]) + ref_diff;
}

hipError_t launch_finish_summary(float* summary, const float* accq, const float* accp, float ref_diff,
                                 int64_t R, int D, int mode, int64_t row_stride, int64_t row_shift, hipStream_t st) {
    if (R == 0) return hipSuccess;
    hipLaunchKernelGGL(k_finish_summary, dim3((unsigned)((R + 255) / 256)), dim3(256), 0, st, summary, accq, accp, ref_diff,
                       R, D, mode, row_stride, row_shift);
    return hipGetLastError();
}

// tokens [G, gamma+1, D]: groups with n_accept == gamma also emit the bonus token (Alg. 1, last line)
__global__ void k_append_bonus(float* __restrict__ tokens, int32_t* __restrict__ n_out, const int32_t* __restrict__ n_accept,
                               const float* __restrict__ bonus, int64_t G, int gamma, int D) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t g = i / D; const int d = (int)(i % D);
    if (g >= G || n_accept[g] != gamma) return;
    tokens[(g * (gamma + 1) + gamma) * D + d] = bonus[g * D + d];
    if (d == 0) n_out[g] = gamma + 1;
}

hipError_t launch_append_bonus(float* tokens, int32_t* n_out, const int32_t* n_accept, const float* bonus,
                               int64_t G, int gamma, int D, hipStream_t st) {
    if (G == 0) return hipSuccess;
    hipLaunchKernelGGL(k_append_bonus, dim3((unsigned)((G * D + 255) / 256)), dim3(256), 0, st, tokens, n_out, n_accept, bonus, G, gamma, D);
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
