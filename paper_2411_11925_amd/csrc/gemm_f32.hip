// fp32 GEMM C[M,N] = epilogue(A[M,K] * B[N,K]^T + bias) on the vector ALUs.
// This is the CSD_F32 path: every product and sum in fp32 (fused multiply-add),
// used for parity against the fp64 oracle at 1e-4.  64x64 tile per workgroup,
// 4x4 outputs per thread, K walked in slabs of 16 through LDS.
// Requirements (checked by the caller): N % 64 == 0, K % 4 == 0; M is free.
#include "internal.hpp"

namespace csd {

namespace {
constexpr int BM = 64, BN = 64, BK = 16, PAD = 4;

__device__ __forceinline__ float silu_acc(float a) { return a / (1.0f + expf(-a)); }

template <int EPI>
__global__ __launch_bounds__(256) void k_gemm_f32(const float* __restrict__ A, int lda, const float* __restrict__ B,
                                                  const float* __restrict__ bias, float* __restrict__ C, int ldc,
                                                  const float* __restrict__ gate, int ldg, int M, int N, int K) {
    __shared__ float As[BK][BM + PAD];
    __shared__ float Bs[BK][BN + PAD];
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t m0 = (int64_t)blockIdx.y * BM;
    const int n0 = blockIdx.x * BN;
    const int lrow = tid >> 2;            // 0..63: tile row this thread stages
    const int lk = (tid & 3) * 4;         // 0,4,8,12: first k of its float4
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

    for (int k0 = 0; k0 < K; k0 += BK) {
        float4 av = make_float4(0.f, 0.f, 0.f, 0.f), bv = av;
        if (k0 + lk < K) {
            if (m0 + lrow < M) av = *reinterpret_cast<const float4*>(A + (m0 + lrow) * lda + k0 + lk);
            bv = *reinterpret_cast<const float4*>(B + (size_t)(n0 + lrow) * K + k0 + lk);
        }
        __syncthreads();
        As[lk + 0][lrow] = av.x; As[lk + 1][lrow] = av.y; As[lk + 2][lrow] = av.z; As[lk + 3][lrow] = av.w;
        Bs[lk + 0][lrow] = bv.x; Bs[lk + 1][lrow] = bv.y; Bs[lk + 2][lrow] = bv.z; Bs[lk + 3][lrow] = bv.w;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            const float4 a4 = *reinterpret_cast<const float4*>(&As[k][ty * 4]);
            const float4 b4 = *reinterpret_cast<const float4*>(&Bs[k][tx * 4]);
            const float a[4] = {a4.x, a4.y, a4.z, a4.w};
            const float b[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
    }
    const int n = n0 + tx * 4;
    const float4 bb = *reinterpret_cast<const float4*>(bias + n);
    const float bj[4] = {bb.x, bb.y, bb.z, bb.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t m = m0 + ty * 4 + i;
        if (m >= M) continue;
        float v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = acc[i][j] + bj[j];
        float* cp = C + m * ldc + n;
        if (EPI == EPI_BIAS_SILU) {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = silu_acc(v[j]);
        } else if (EPI == EPI_GATE_RES) {
            const float4 g = *reinterpret_cast<const float4*>(gate + m * ldg + n);
            const float4 c = *reinterpret_cast<const float4*>(cp);
            v[0] = fmaf(g.x, v[0], c.x); v[1] = fmaf(g.y, v[1], c.y);
            v[2] = fmaf(g.z, v[2], c.z); v[3] = fmaf(g.w, v[3], c.w);
        }
        *reinterpret_cast<float4*>(cp) = make_float4(v[0], v[1], v[2], v[3]);
    }
}
}  // namespace

hipError_t launch_gemm_f32(const GemmArgs& g, hipStream_t st) {
    if (g.M == 0) return hipSuccess;
    if (g.N % BN != 0 || g.K % 4 != 0 || g.lda % 4 != 0 || g.ldc % 4 != 0) return hipErrorInvalidValue;
    const int64_t mt = ((int64_t)g.M + BM - 1) / BM;
    if (mt > 65535) return hipErrorInvalidValue;
    dim3 grid(g.N / BN, (unsigned)mt), block(256);
    const float* A = (const float*)g.A; const float* B = (const float*)g.B; float* C = (float*)g.C;
    const float* gate = (const float*)g.gate;
    switch (g.epi) {
        case EPI_BIAS: hipLaunchKernelGGL(k_gemm_f32<EPI_BIAS>, grid, block, 0, st, A, g.lda, B, g.bias, C, g.ldc, gate, g.ldg, g.M, g.N, g.K); break;
        case EPI_BIAS_SILU: hipLaunchKernelGGL(k_gemm_f32<EPI_BIAS_SILU>, grid, block, 0, st, A, g.lda, B, g.bias, C, g.ldc, gate, g.ldg, g.M, g.N, g.K); break;
        case EPI_GATE_RES:
            if (g.ldg % 4 != 0) return hipErrorInvalidValue;
            hipLaunchKernelGGL(k_gemm_f32<EPI_GATE_RES>, grid, block, 0, st, A, g.lda, B, g.bias, C, g.ldc, gate, g.ldg, g.M, g.N, g.K); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace csd
