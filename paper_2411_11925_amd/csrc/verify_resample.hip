// Accept test with first-reject scan (Alg. 1; Eq. 7) and acceptance-rejection
// resampling from max(0, p - q)/Z with the threshold of Corollary 1 (Sec. 3.3).
//
// Layout of the work: a row has D <= 16 coordinates, so a 64-lane wavefront is cut
// into S = 64/D segments of D lanes.  Verify gives each segment one row of the
// group; resample gives each segment one TRIAL, so S proposals of the
// repeat-until loop are evaluated together and the first accepted one (in trial
// order) wins - the same result as the sequential loop, in 1/S of the passes.
#include "internal.hpp"
#include "rng.hpp"

namespace csd {

namespace {

template <int D>
__device__ __forceinline__ float seg_sum(float v) {
#pragma unroll
    for (int o = D / 2; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// one wave per group
template <int D>
__global__ __launch_bounds__(256) void k_verify(const float* __restrict__ summary, int64_t G, int gamma,
                                                uint64_t seed, uint64_t row_offset, float tau,
                                                int32_t* __restrict__ n_accept, float* __restrict__ log_ratio,
                                                uint8_t* __restrict__ mask) {
    constexpr int S = 64 / D, SW = 5 * D + 1;
    const int lane = threadIdx.x & 63;
    const int64_t g = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (g >= G) return;
    const int seg = lane / D, d = lane % D;
    const float inv_tau = 1.0f / tau;
    int first_reject = gamma;
    for (int i0 = 0; i0 < gamma; i0 += S) {
        const int i = i0 + seg;
        bool accept = true;           // rows past the group's end never reject
        if (i < gamma) {
            const int64_t r = g * gamma + i;
            const float* s = summary + r * SW;
            const float mu_p = s[d], lv_p = s[D + d], mu_q = s[2 * D + d], lv_q = s[3 * D + d], x0 = s[4 * D + d];
            const float zp = (x0 - mu_p) * expf(-0.5f * lv_p) * inv_tau;
            const float zq = (x0 - mu_q) * expf(-0.5f * lv_q) * inv_tau;
            // log N(x0;mu_p,.) - log N(x0;mu_q,.) per coordinate (log tau and log 2 pi cancel)
            const float term = 0.5f * ((zq - zp) * (zq + zp) + (lv_q - lv_p));   // zq^2 - zp^2, exactly 0 for equal models
            float ell = seg_sum<D>(term) + s[5 * D];
            const float u = uniform_at(seed, row_offset + (uint64_t)r, 0u, CSD_STREAM_ACCEPT_U);
            accept = logf(u) <= ell;                     // NaN compares false: reject
            if (d == 0) {
                if (log_ratio) log_ratio[r] = ell;
                if (mask) mask[r] = accept ? 1 : 0;
            }
        }
        const unsigned long long rej = __ballot(!accept);   // D equal bits per segment
        if (rej != 0ull && first_reject == gamma) first_reject = i0 + (__ffsll((long long)rej) - 1) / D;
    }
    if (lane == 0) n_accept[g] = first_reject;
}

// one wave per group
template <int D>
__global__ __launch_bounds__(256) void k_resample(const float* __restrict__ summary, const int32_t* __restrict__ n_accept,
                                                  int64_t G, int gamma, uint64_t seed, uint64_t row_offset, float tau,
                                                  int max_trips, float* __restrict__ tokens, int32_t* __restrict__ n_out,
                                                  int32_t* __restrict__ trips, uint32_t* __restrict__ flags) {
    constexpr int S = 64 / D, SW = 5 * D + 1;
    const int lane = threadIdx.x & 63;
    const int64_t g = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (g >= G) return;
    int n = n_accept[g];
    n = n < 0 ? 0 : (n > gamma ? gamma : n);
    float* tok = tokens + g * (int64_t)(gamma + 1) * D;
    // emit x_1..x_n and clear the rest
    for (int e = lane; e < (gamma + 1) * D; e += 64) {
        const int i = e / D, d = e % D;
        tok[e] = (i < n) ? summary[(g * gamma + i) * SW + 4 * D + d] : 0.f;
    }
    if (n >= gamma) {
        if (lane == 0) { n_out[g] = gamma; if (trips) trips[g] = 0; if (flags) flags[g] = 0u; }
        return;
    }
    const int seg = lane / D, d = lane % D;
    const int64_t r = g * gamma + n;                       // first rejected row
    const uint64_t grow = row_offset + (uint64_t)r;
    const float* s = summary + r * SW;
    const float mu_p = s[d], lv_p = s[D + d], mu_q = s[2 * D + d], lv_q = s[3 * D + d];
    const float log_sigma = s[5 * D];
    const float sd_p = tau * expf(0.5f * lv_p);
    const float inv_sd_q = expf(-0.5f * lv_q) / tau;
    uint32_t fl = 0u;
    int used = 0;
    float xp = 0.f;
    bool done = false;
    for (int k0 = 0; k0 < max_trips && !done; k0 += S) {
        const int k = k0 + seg;
        const bool live = k < max_trips;
        float nrm[4];
        normals4(seed, grow, (uint32_t)k, CSD_STREAM_RESAMPLE_N, (uint32_t)(d >> 2), nrm);
        const float e = nrm[d & 3];
        xp = fmaf(sd_p, e, mu_p);                          // x' ~ p(.|x_1^p)
        const float zq = (xp - mu_q) * inv_sd_q;
        // log q(x') - log p(x') per coordinate; (x'-mu_p)/sd_p is e itself
        const float term = 0.5f * ((e - zq) * (e + zq) + (lv_p - lv_q));
        const float a = seg_sum<D>(term) - log_sigma;
        float alpha_s = (a < 0.f) ? -expm1f(a) : 0.f;      // max(0, 1 - exp(a)); NaN -> 0
        const bool nan = (a != a);
        const float u = uniform_at(seed, grow, (uint32_t)k, CSD_STREAM_RESAMPLE_U);
        const bool ok = live && (u <= alpha_s);
        const unsigned long long okb = __ballot(ok);
        const unsigned long long nanb = __ballot(live && nan);
        int last_seg;                                      // segment whose proposal is kept
        if (okb != 0ull) {
            last_seg = (__ffsll((long long)okb) - 1) / D;
            done = true;
        } else {
            const int live_segs = (max_trips - k0 < S) ? (max_trips - k0) : S;
            last_seg = live_segs - 1;
        }
        used = k0 + last_seg + 1;
        // NaNs met in the trials actually taken (up to and including last_seg)
        const unsigned long long upto = (last_seg + 1) * D >= 64 ? ~0ull : ((1ull << ((last_seg + 1) * D)) - 1ull);
        if (nanb & upto) fl |= CSD_FLAG_NONFINITE;
        if (seg == last_seg && (done || used >= max_trips)) tok[n * D + d] = xp;
    }
    if (!done) fl |= CSD_FLAG_CAP;
    if (lane == 0) { n_out[g] = n + 1; if (trips) trips[g] = used; if (flags) flags[g] = fl; }
}

}  // namespace

hipError_t launch_verify(const float* summary, int64_t G, int gamma, int D, uint64_t seed, uint64_t row_offset,
                         float tau, int32_t* n_accept, float* log_ratio, uint8_t* mask, hipStream_t st) {
    if (G == 0) return hipSuccess;
    dim3 grid((unsigned)((G + 3) / 4)), block(256);
    switch (D) {
        case 4: hipLaunchKernelGGL(k_verify<4>, grid, block, 0, st, summary, G, gamma, seed, row_offset, tau, n_accept, log_ratio, mask); break;
        case 8: hipLaunchKernelGGL(k_verify<8>, grid, block, 0, st, summary, G, gamma, seed, row_offset, tau, n_accept, log_ratio, mask); break;
        case 16: hipLaunchKernelGGL(k_verify<16>, grid, block, 0, st, summary, G, gamma, seed, row_offset, tau, n_accept, log_ratio, mask); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_resample(const float* summary, const int32_t* n_accept, int64_t G, int gamma, int D,
                           uint64_t seed, uint64_t row_offset, float tau, int max_trips,
                           float* tokens, int32_t* n_out, int32_t* trips, uint32_t* flags, hipStream_t st) {
    if (G == 0) return hipSuccess;
    dim3 grid((unsigned)((G + 3) / 4)), block(256);
    switch (D) {
        case 4: hipLaunchKernelGGL(k_resample<4>, grid, block, 0, st, summary, n_accept, G, gamma, seed, row_offset, tau, max_trips, tokens, n_out, trips, flags); break;
        case 8: hipLaunchKernelGGL(k_resample<8>, grid, block, 0, st, summary, n_accept, G, gamma, seed, row_offset, tau, max_trips, tokens, n_out, trips, flags); break;
        case 16: hipLaunchKernelGGL(k_resample<16>, grid, block, 0, st, summary, n_accept, G, gamma, seed, row_offset, tau, max_trips, tokens, n_out, trips, flags); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace csd
