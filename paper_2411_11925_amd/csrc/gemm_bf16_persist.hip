// Persistent bf16 GEMM for the large layers: C[M,N] = act(A[M,K] * B[N,K]^T + bias), bf16 out.
//
// Same tile machinery as gemm_bf16.hip (256x256 tile, K slabs of 64 loaded straight into
// XOR-swizzled LDS, 32x32x16 MFMAs, weights as the MFMA "A" operand), with two changes
// that take the epilogue off the critical path:
//   * one workgroup per CU walks a list of tiles, so the first slab of the next tile is
//     already in flight while the current tile finishes;
//   * a finished tile is converted to packed bf16 in registers (4 waves x 128x128, one
//     wave per SIMD, leaves room for that) and its stores are TRICKLED out, one 32x32
//     block per K slab of the next tile.  HBM sees a steady write stream instead of a
//     burst from all CUs at once, and no wave ever waits for a store.
// The stores are inline `global_store_dwordx2` so that their number between two direct
// loads is exact: vmcnt counts loads and stores in issue order, so "slab landed" is
// vmcnt <= (stores issued after that slab's loads).  p.safe_wait makes every wait a
// vmcnt(0) (no overlap) - the two modes must give identical results.
// Requirements: K % 64 == 0, N % 256 == 0, 16-byte aligned A, B, C and leading dims.
#include <type_traits>

#include "internal.hpp"

namespace csd {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BM = 256, BN = 256, BK = 64, WN = 2, NW = 4;
constexpr int TM = 128, TN = 128, FM = 4, FN = 4;
constexpr int ROW_B = BK * 2, STAGE_B = (BM + BN) * ROW_B;
constexpr int GPW = (BM + BN) / 8 / NW;     // direct loads per wave and slab (16)
constexpr int NPIECE = FM * FN;             // one 32x32 block per piece
constexpr int SPP = 4;                      // stores per piece (q = 0..3)

struct PParams {
    const bf16_t* A; int lda;
    const bf16_t* B;
    const float* bias;
    bf16_t* C; int ldc;
    int M, N, K;
    int tiles_m, tiles_n;
    int safe_wait;
};

__device__ __forceinline__ float silu_fast(float a) { return a / (1.0f + __expf(-a)); }

template <int N> __device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

__device__ __forceinline__ void store8(bf16_t* ptr, uint32_t lo, uint32_t hi) {
    const unsigned long long v = (unsigned long long)lo | ((unsigned long long)hi << 32);
    asm volatile("global_store_dwordx2 %0, %1, off" ::"v"(ptr), "v"(v) : "memory");
}

template <int EPI>
__global__ __launch_bounds__(256) void k_gemm_bf16_persist(PParams p) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, khalf = lane >> 5;

    // ---- tiles of this workgroup.  Ids sharing id%8 sit on one XCD: they take consecutive
    // tiles (n fastest) of that XCD's slice, so the A rows in flight are shared through L2.
    const int total = p.tiles_m * p.tiles_n;
    const int nwg = gridDim.x, wg = blockIdx.x;
    int my_tiles, tile0, tstride;
    if ((total % 8 == 0) && (nwg % 8 == 0)) {
        const int per_xcd = total / 8, slots = nwg / 8, slot = wg / 8;
        my_tiles = slot < per_xcd ? (per_xcd - slot + slots - 1) / slots : 0;
        tile0 = (wg % 8) * per_xcd + slot; tstride = slots;
    } else {
        my_tiles = wg < total ? (total - wg + nwg - 1) / nwg : 0;
        tile0 = wg; tstride = nwg;
    }
    auto tile_of = [&](int it) { return tile0 + it * tstride; };

    // ---- loader (see gemm_bf16.hip)
    const int lr = lane >> 3, pc = lane & 7;
    const int ld_chunk = pc ^ ((((wave & 1) << 2) + (lr >> 1)) & 7);
    auto issue_loads = [&](int stage, int tile, int k0) {
        const int64_t m0 = (int64_t)(tile / p.tiles_n) * BM;
        const int n0 = (tile % p.tiles_n) * BN;
#pragma unroll
        for (int i = 0; i < GPW; ++i) {
            const int g = wave + i * NW;
            const int row = g * 8 + lr;
            const bf16_t* src;
            if (g < BM / 8) {
                int64_t r = m0 + row;
                r = r < p.M ? r : (int64_t)p.M - 1;
                src = p.A + r * p.lda + k0 + ld_chunk * 8;
            } else {
                src = p.B + (size_t)(n0 + row - BM) * p.K + k0 + ld_chunk * 8;
            }
            __builtin_amdgcn_global_load_lds(src, (__attribute__((address_space(3))) void*)(smem + stage * STAGE_B + g * 1024),
                                             16, 0, 0);
        }
    };

    const int swz = (l32 >> 1) & 7;
    int koff[BK / 16];
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) koff[kk] = ((kk * 2 + khalf) ^ swz) * 16;
    const int a_row_off = (wm * TM + l32) * ROW_B;
    const int b_row_off = (BM + wn * TN + l32) * ROW_B;

    f32x16 acc[FM][FN];
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    uint32_t pend[NPIECE][SPP][2];       // finished tile, packed bf16, waiting to be stored
    bf16_t* pend_ptr = nullptr;          // &C[row of this lane in block row 0][first feature of this lane]
    bool have_pend = false;
    int prev_stores = 0;                 // inline stores issued after the latest direct loads (0 or SPP)

    auto store_piece = [&](auto piece_c) {
        constexpr int u = decltype(piece_c)::value;
        constexpr int i = u / FN, j = u % FN;
        bf16_t* base = pend_ptr + (size_t)i * 32 * p.ldc + j * 32;
#pragma unroll
        for (int q = 0; q < SPP; ++q) store8(base + q * 8, pend[u][q][0], pend[u][q][1]);
    };

    const int nk = p.K / BK;
    int gs = 0;                          // slabs done so far (stage = gs & 1)
    if (my_tiles > 0) issue_loads(0, tile_of(0), 0);

    auto slab = [&](int it, int kt) {
        if (prev_stores && !p.safe_wait) wait_vmcnt<SPP>(); else wait_vmcnt<0>();
        prev_stores = 0;
        __syncthreads();
        if (kt + 1 < nk) issue_loads((gs + 1) & 1, tile_of(it), (kt + 1) * BK);
        else if (it + 1 < my_tiles) issue_loads((gs + 1) & 1, tile_of(it + 1), 0);
        const unsigned char* sa = smem + (gs & 1) * STAGE_B + a_row_off;
        const unsigned char* sb = smem + (gs & 1) * STAGE_B + b_row_off;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            bf16x8 fa[FM], fb[FN];
#pragma unroll
            for (int i = 0; i < FM; ++i)
                fa[i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(sa + i * 32 * ROW_B + koff[kk]));
#pragma unroll
            for (int j = 0; j < FN; ++j)
                fb[j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(sb + j * 32 * ROW_B + koff[kk]));
#pragma unroll
            for (int i = 0; i < FM; ++i)
#pragma unroll
                for (int j = 0; j < FN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
        }
        ++gs;
    };

    for (int it = 0; it < my_tiles; ++it) {
        // K slabs 0..14 each carry one piece (1..15) of the previous tile; piece 0 went out
        // right after the conversion below
#define CSD_SLAB_WITH_PIECE(U)                                                                   \
        if (U < nk) {                                                                            \
            slab(it, U);                                                                         \
            if (have_pend && U + 1 < NPIECE) { store_piece(std::integral_constant<int, U + 1>{}); prev_stores = SPP; } \
        }
        CSD_SLAB_WITH_PIECE(0) CSD_SLAB_WITH_PIECE(1) CSD_SLAB_WITH_PIECE(2) CSD_SLAB_WITH_PIECE(3)
        CSD_SLAB_WITH_PIECE(4) CSD_SLAB_WITH_PIECE(5) CSD_SLAB_WITH_PIECE(6) CSD_SLAB_WITH_PIECE(7)
        CSD_SLAB_WITH_PIECE(8) CSD_SLAB_WITH_PIECE(9) CSD_SLAB_WITH_PIECE(10) CSD_SLAB_WITH_PIECE(11)
        CSD_SLAB_WITH_PIECE(12) CSD_SLAB_WITH_PIECE(13) CSD_SLAB_WITH_PIECE(14)
#undef CSD_SLAB_WITH_PIECE
        for (int kt = 15; kt < nk; ++kt) slab(it, kt);
        // pieces that found no slab (K < 15*64): out now
        if (have_pend) {
#define CSD_FLUSH(U) if (U > nk) store_piece(std::integral_constant<int, U>{});
            CSD_FLUSH(1) CSD_FLUSH(2) CSD_FLUSH(3) CSD_FLUSH(4) CSD_FLUSH(5) CSD_FLUSH(6) CSD_FLUSH(7) CSD_FLUSH(8)
            CSD_FLUSH(9) CSD_FLUSH(10) CSD_FLUSH(11) CSD_FLUSH(12) CSD_FLUSH(13) CSD_FLUSH(14) CSD_FLUSH(15)
#undef CSD_FLUSH
            if (nk < NPIECE - 1) prev_stores = 0;      // unknown count: next wait drains everything
        }
        // ---- tile done: bias, activation, pack; restart the accumulators
        const int tile = tile_of(it);
        const int64_t m0 = (int64_t)(tile / p.tiles_n) * BM;
        const int n0 = (tile % p.tiles_n) * BN;
        const bool full = m0 + BM <= p.M;
#pragma unroll
        for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn * TN + j * 32 + q * 8 + khalf * 4;
                const float4 bb = *reinterpret_cast<const float4*>(p.bias + n);
#pragma unroll
                for (int i = 0; i < FM; ++i) {
                    float v0 = acc[i][j][4 * q + 0] + bb.x, v1 = acc[i][j][4 * q + 1] + bb.y;
                    float v2 = acc[i][j][4 * q + 2] + bb.z, v3 = acc[i][j][4 * q + 3] + bb.w;
                    if (EPI == EPI_BIAS_SILU) { v0 = silu_fast(v0); v1 = silu_fast(v1); v2 = silu_fast(v2); v3 = silu_fast(v3); }
                    pend[i * FN + j][q][0] = pack_bf16x2(v0, v1);
                    pend[i * FN + j][q][1] = pack_bf16x2(v2, v3);
                }
                asm volatile("" ::: "memory");     // keep the bias loads from piling up in registers
            }
#pragma unroll
        for (int i = 0; i < FM; ++i)
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
        pend_ptr = p.C + (m0 + wm * TM + l32) * p.ldc + n0 + wn * TN + khalf * 4;
        if (full) {
            have_pend = true;
            store_piece(std::integral_constant<int, 0>{});
            prev_stores = (nk < NPIECE - 1) ? 0 : SPP;
        } else {
            // ragged last row of tiles: predicated stores right away, nothing left pending
            have_pend = false;
            prev_stores = 0;
#pragma unroll
            for (int i = 0; i < FM; ++i) {
                if (m0 + wm * TM + i * 32 + l32 < p.M) {
#pragma unroll
                    for (int j = 0; j < FN; ++j)
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            *reinterpret_cast<uint2*>(pend_ptr + (size_t)i * 32 * p.ldc + j * 32 + q * 8) =
                                make_uint2(pend[i * FN + j][q][0], pend[i * FN + j][q][1]);
                }
            }
        }
    }
    if (have_pend) {
#define CSD_FLUSH(U) store_piece(std::integral_constant<int, U>{});
        CSD_FLUSH(1) CSD_FLUSH(2) CSD_FLUSH(3) CSD_FLUSH(4) CSD_FLUSH(5) CSD_FLUSH(6) CSD_FLUSH(7) CSD_FLUSH(8)
        CSD_FLUSH(9) CSD_FLUSH(10) CSD_FLUSH(11) CSD_FLUSH(12) CSD_FLUSH(13) CSD_FLUSH(14) CSD_FLUSH(15)
#undef CSD_FLUSH
    }
}

int num_cus() {
    static int n = 0;
    if (n == 0) {
        int dev = 0; hipDeviceProp_t pr;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&pr, dev) == hipSuccess) n = pr.multiProcessorCount;
        if (n <= 0) n = 256;
    }
    return n;
}

}  // namespace

hipError_t launch_gemm_bf16_persist(const GemmArgs& g, hipStream_t st, int safe_wait) {
    if (g.M == 0) return hipSuccess;
    if (g.K % BK != 0 || g.N % BN != 0 || g.lda % 8 != 0 || g.ldc % 4 != 0 || g.c_is_f32) return hipErrorInvalidValue;
    if (((uintptr_t)g.A & 15u) || ((uintptr_t)g.B & 15u) || ((uintptr_t)g.C & 15u)) return hipErrorInvalidValue;
    if (g.epi != EPI_BIAS && g.epi != EPI_BIAS_SILU) return hipErrorInvalidValue;
    PParams p;
    p.A = (const bf16_t*)g.A; p.lda = g.lda; p.B = (const bf16_t*)g.B; p.bias = g.bias;
    p.C = (bf16_t*)g.C; p.ldc = g.ldc; p.M = g.M; p.N = g.N; p.K = g.K;
    p.tiles_m = (g.M + BM - 1) / BM; p.tiles_n = g.N / BN; p.safe_wait = safe_wait;
    const int total = p.tiles_m * p.tiles_n;
    int grid = num_cus() < total ? num_cus() : total;
    const size_t smem = (size_t)2 * STAGE_B;
    static bool attr_done = false;
    if (!attr_done) {
        hipError_t e = hipFuncSetAttribute((const void*)k_gemm_bf16_persist<EPI_BIAS>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        e = hipFuncSetAttribute((const void*)k_gemm_bf16_persist<EPI_BIAS_SILU>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_done = true;
    }
    if (g.epi == EPI_BIAS) hipLaunchKernelGGL(k_gemm_bf16_persist<EPI_BIAS>, dim3(grid), dim3(256), smem, st, p);
    else hipLaunchKernelGGL(k_gemm_bf16_persist<EPI_BIAS_SILU>, dim3(grid), dim3(256), smem, st, p);
    return hipGetLastError();
}

}  // namespace csd
