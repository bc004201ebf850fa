// Mixture-of-Gaussians output heads (the paper's appendix on other forms of the output
// distribution): p(x) = sum_k pi_k N(x; mu_k, Sigma_k) with diagonal Sigma_k.  The densities
// are explicit, so the accept test of Alg. 1 uses p(x)/q(x) itself and the modified
// distribution max(0, p - q)/Z is sampled by acceptance-rejection with proposal p and
// threshold max(0, p(x) - q(x))/p(x).
//
// Layout of the work as in the Gaussian case: a row has D <= 16 coordinates, a 64-lane
// wavefront is cut into S = 64/D segments of D lanes; verify gives each segment one row of
// the group, resample gives each segment one trial.  A mixture is (pi [R,K], mu [R,K,D],
// logvar [R,K,D]); pi >= 0 need not sum to 1.
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

// log sum_k (pi_k / sum pi) N(x; mu_k, .) up to the constant -D/2 log(2 pi), which cancels in
// every ratio taken here.  x is this lane's coordinate d of the point; the result is the same
// in all D lanes of the segment.  Running log-sum-exp over the components with pi_k > 0.
template <int D>
__device__ __forceinline__ float mix_logpdf(float x, const float* __restrict__ pi, const float* __restrict__ mu,
                                            const float* __restrict__ lv, int K, int d) {
    float total = 0.f, m = -INFINITY, s = 0.f;
    for (int k = 0; k < K; ++k) {
        const float w = pi[k];
        total += w;
        const float l = lv[k * D + d], z = (x - mu[k * D + d]);
        const float c = seg_sum<D>(-0.5f * fmaf(z * z, expf(-l), l));
        if (w > 0.f) {
            const float a = c + logf(w);
            if (a > m) { s = s * expf(m - a) + 1.f; m = a; }      // exp(-inf) = 0 on the first component
            else s += expf(a - m);
        }
    }
    return m + logf(s) - logf(total);
}

// first k whose running sum of pi (fp32, left to right) reaches u * sum(pi)
__device__ __forceinline__ int mix_pick(const float* __restrict__ pi, int K, float u) {
    float total = 0.f;
    for (int k = 0; k < K; ++k) total += pi[k];
    const float thr = u * total;
    float run = 0.f;
    for (int k = 0; k < K; ++k) {
        run += pi[k];
        if (run >= thr) return k;
    }
    return K - 1;
}

// x_i ~ q_i: one segment of D lanes per row
template <int D>
__global__ __launch_bounds__(256) void k_gmm_draft_sample(const float* __restrict__ pi, const float* __restrict__ mu,
                                                          const float* __restrict__ lv, int64_t R, int K, uint64_t seed,
                                                          uint64_t row_offset, float* __restrict__ x) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t r = i / D;
    const int d = (int)(i % D);
    if (r >= R) return;
    const uint64_t grow = row_offset + (uint64_t)r;
    const int k = mix_pick(pi + r * K, K, uniform_at(seed, grow, 0u, CSD_STREAM_GMM_PICK));
    float nrm[4];
    normals4(seed, grow, 0u, CSD_STREAM_TRAJ, (uint32_t)(d >> 2), nrm);
    const int64_t o = (r * K + k) * D + d;
    x[r * D + d] = fmaf(expf(0.5f * lv[o]), nrm[d & 3], mu[o]);
}

struct Mix { const float* pi; const float* mu; const float* lv; };

// The accept test reads both mixtures of every row once and is bound by HBM, so its lanes are
// laid out for wide loads: a team of L lanes takes one row, L/(D/4) components at a time, each
// lane 4 consecutive coordinates of one component (one 16-byte load of mu and of logvar).  A
// component's exponent is summed over its D/4 lanes, the log-sum-exp over the team.
// L = the power of two >= K*D/4, at most 16; 64/L rows of the group per pass.  One wave per group.
template <int D>
__device__ __forceinline__ float team_logpdf(const float4 x4, const float* __restrict__ pi, const float* __restrict__ mu,
                                             const float* __restrict__ lv, int K, int L, int t) {
    constexpr int PD = D / 4;                    // lanes per component
    const int kc = t / PD, d0 = (t % PD) * 4, CK = L / PD;
    float total = 0.f;
    for (int k = 0; k < K; ++k) total += pi[k];
    float m = -INFINITY, s = 0.f;
    for (int k0 = 0; k0 < K; k0 += CK) {
        const int k = k0 + kc;
        const bool valid = k < K;
        const int kk = valid ? k : K - 1;
        const float4 m4 = *reinterpret_cast<const float4*>(mu + kk * D + d0);
        const float4 l4 = *reinterpret_cast<const float4*>(lv + kk * D + d0);
        const float w = pi[kk];
        const float z0 = x4.x - m4.x, z1 = x4.y - m4.y, z2 = x4.z - m4.z, z3 = x4.w - m4.w;
        float c = fmaf(z0 * z0, expf(-l4.x), l4.x) + fmaf(z1 * z1, expf(-l4.y), l4.y) +
                  fmaf(z2 * z2, expf(-l4.z), l4.z) + fmaf(z3 * z3, expf(-l4.w), l4.w);
#pragma unroll
        for (int o = PD / 2; o >= 1; o >>= 1) c += __shfl_xor(c, o, 64);
        const float a = (valid && w > 0.f) ? fmaf(-0.5f, c, logf(w)) : -INFINITY;
        float mc = a;                            // maximum over the team's components of this chunk
        for (int o = L / 2; o >= 1; o >>= 1) mc = fmaxf(mc, __shfl_xor(mc, o, 64));
        if (mc > -INFINITY) {                    // (uniform over the team)
            float e = (t % PD == 0 && a > -INFINITY) ? expf(a - mc) : 0.f;    // one lane per component adds
            for (int o = L / 2; o >= 1; o >>= 1) e += __shfl_xor(e, o, 64);
            if (mc > m) { s = s * expf(m - mc) + e; m = mc; }
            else s += e * expf(mc - m);
        }
    }
    return m + logf(s) - logf(total);
}

template <int D>
__global__ __launch_bounds__(256) void k_gmm_verify(const float* __restrict__ x, Mix p, Mix q, int64_t G, int gamma, int K,
                                                    int L, uint64_t seed, uint64_t row_offset,
                                                    int32_t* __restrict__ n_accept, float* __restrict__ log_ratio,
                                                    uint8_t* __restrict__ mask) {
    const int lane = threadIdx.x & 63;
    const int64_t g = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (g >= G) return;
    const int RPW = 64 / L, team = lane / L, t = lane % L;
    int first_reject = gamma;
    for (int i0 = 0; i0 < gamma; i0 += RPW) {
        const int i = i0 + team;
        // teams past the group's end evaluate its last row (the shuffles need all lanes) and never reject
        const int64_t r = g * gamma + (i < gamma ? i : gamma - 1);
        const float4 x4 = *reinterpret_cast<const float4*>(x + r * D + (t % (D / 4)) * 4);
        const float ell = team_logpdf<D>(x4, p.pi + r * K, p.mu + r * K * D, p.lv + r * K * D, K, L, t) -
                          team_logpdf<D>(x4, q.pi + r * K, q.mu + r * K * D, q.lv + r * K * D, K, L, t);
        const float u = uniform_at(seed, row_offset + (uint64_t)r, 0u, CSD_STREAM_ACCEPT_U);
        const bool accept = (i >= gamma) || (logf(u) <= ell);            // NaN compares false: reject
        if (i < gamma && t == 0) {
            if (log_ratio) log_ratio[r] = ell;
            if (mask) mask[r] = accept ? 1 : 0;
        }
        const unsigned long long rej = __ballot(!accept);                // L equal bits per team
        if (rej != 0ull && first_reject == gamma) first_reject = i0 + (__ffsll((long long)rej) - 1) / L;
    }
    if (lane == 0) n_accept[g] = first_reject;
}

// one wave per group; S trials of the repeat-until loop per pass, the first accepted one wins
template <int D>
__global__ __launch_bounds__(256) void k_gmm_resample(const float* __restrict__ x, const int32_t* __restrict__ n_accept,
                                                      Mix p, Mix q, int64_t G, int gamma, int K, uint64_t seed,
                                                      uint64_t row_offset, int max_trips, float* __restrict__ tokens,
                                                      int32_t* __restrict__ n_out, int32_t* __restrict__ trips,
                                                      uint32_t* __restrict__ flags) {
    constexpr int S = 64 / D;
    const int lane = threadIdx.x & 63;
    const int64_t g = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (g >= G) return;
    int n = n_accept[g];
    n = n < 0 ? 0 : (n > gamma ? gamma : n);
    float* tok = tokens + g * (int64_t)(gamma + 1) * D;
    for (int e = lane; e < (gamma + 1) * D; e += 64) {
        const int i = e / D, d = e % D;
        tok[e] = (i < n) ? x[(g * gamma + i) * D + d] : 0.f;
    }
    if (n >= gamma) {
        if (lane == 0) { n_out[g] = gamma; if (trips) trips[g] = 0; if (flags) flags[g] = 0u; }
        return;
    }
    const int seg = lane / D, d = lane % D;
    const int64_t r = g * gamma + n;                       // first rejected row
    const uint64_t grow = row_offset + (uint64_t)r;
    const float* ppi = p.pi + r * K; const float* pmu = p.mu + r * K * D; const float* plv = p.lv + r * K * D;
    const float* qpi = q.pi + r * K; const float* qmu = q.mu + r * K * D; const float* qlv = q.lv + r * K * D;
    uint32_t fl = 0u;
    int used = 0;
    bool done = false;
    for (int k0 = 0; k0 < max_trips && !done; k0 += S) {
        const int k = k0 + seg;
        const bool live = k < max_trips;
        const int c = mix_pick(ppi, K, uniform_at(seed, grow, (uint32_t)(1 + k), CSD_STREAM_GMM_PICK));
        float nrm[4];
        normals4(seed, grow, (uint32_t)k, CSD_STREAM_RESAMPLE_N, (uint32_t)(d >> 2), nrm);
        const float xp = fmaf(expf(0.5f * plv[c * D + d]), nrm[d & 3], pmu[c * D + d]);      // x' ~ p
        const float a = mix_logpdf<D>(xp, qpi, qmu, qlv, K, d) - mix_logpdf<D>(xp, ppi, pmu, plv, K, d);
        const float alpha_s = (a < 0.f) ? -expm1f(a) : 0.f;              // max(0, 1 - q/p); NaN -> 0
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
        const unsigned long long upto = (last_seg + 1) * D >= 64 ? ~0ull : ((1ull << ((last_seg + 1) * D)) - 1ull);
        if (nanb & upto) fl |= CSD_FLAG_NONFINITE;
        if (seg == last_seg && (done || used >= max_trips)) tok[n * D + d] = xp;
    }
    if (!done) fl |= CSD_FLAG_CAP;
    if (lane == 0) { n_out[g] = n + 1; if (trips) trips[g] = used; if (flags) flags[g] = fl; }
}

}  // namespace

#define CSD_BY_D(KERNEL, GRID, ...)                                                                   \
    switch (D) {                                                                                       \
        case 4: hipLaunchKernelGGL(KERNEL<4>, GRID, dim3(256), 0, st, __VA_ARGS__); break;            \
        case 8: hipLaunchKernelGGL(KERNEL<8>, GRID, dim3(256), 0, st, __VA_ARGS__); break;            \
        case 16: hipLaunchKernelGGL(KERNEL<16>, GRID, dim3(256), 0, st, __VA_ARGS__); break;          \
        default: return hipErrorInvalidValue;                                                          \
    }

hipError_t launch_gmm_draft_sample(const float* pi, const float* mu, const float* lv, int64_t R, int K, int D,
                                   uint64_t seed, uint64_t row_offset, float* x, hipStream_t st) {
    if (R == 0) return hipSuccess;
    const dim3 grid((unsigned)((R * D + 255) / 256));
    CSD_BY_D(k_gmm_draft_sample, grid, pi, mu, lv, R, K, seed, row_offset, x)
    return hipGetLastError();
}

hipError_t launch_gmm_verify(const float* x, const float* pi_p, const float* mu_p, const float* lv_p, const float* pi_q,
                             const float* mu_q, const float* lv_q, int64_t G, int gamma, int K, int D, uint64_t seed,
                             uint64_t row_offset, int32_t* n_accept, float* log_ratio, uint8_t* mask, hipStream_t st) {
    if (G == 0) return hipSuccess;
    const dim3 grid((unsigned)((G + 3) / 4));
    const Mix p{pi_p, mu_p, lv_p}, q{pi_q, mu_q, lv_q};
    // lanes of a row's team: the power of two >= K*D/4, at most 16, so that at least four rows are in
    // flight per wave (one row per wave with 64 lanes was measured: 2.5 against 3.7 TB/s at K = 16)
    int L = D / 4;
    while (L < 16 && L < K * (D / 4)) L *= 2;
    CSD_BY_D(k_gmm_verify, grid, x, p, q, G, gamma, K, L, seed, row_offset, n_accept, log_ratio, mask)
    return hipGetLastError();
}

hipError_t launch_gmm_resample(const float* x, const int32_t* n_accept, const float* pi_p, const float* mu_p,
                               const float* lv_p, const float* pi_q, const float* mu_q, const float* lv_q, int64_t G,
                               int gamma, int K, int D, uint64_t seed, uint64_t row_offset, int max_trips, float* tokens,
                               int32_t* n_out, int32_t* trips, uint32_t* flags, hipStream_t st) {
    if (G == 0) return hipSuccess;
    const dim3 grid((unsigned)((G + 3) / 4));
    const Mix p{pi_p, mu_p, lv_p}, q{pi_q, mu_q, lv_q};
    CSD_BY_D(k_gmm_resample, grid, x, n_accept, p, q, G, gamma, K, seed, row_offset, max_trips, tokens, n_out, trips, flags)
    return hipGetLastError();
}
#undef CSD_BY_D

}  // namespace csd
