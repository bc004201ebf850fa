// bf16 GEMM on the gfx950 matrix cores: C[M,N] = epilogue(A[M,K] * B[N,K]^T + bias),
// A = activations, B = weights ([out,in] row-major), fp32 accumulation.
//
// One workgroup owns a BM x BN tile of C and walks K in slabs of BK = 64.  Each slab
// of A and B goes from global memory STRAIGHT INTO LDS (global_load_lds, 16 bytes per
// lane, no staging registers), double-buffered: the loads of slab k+1 are in flight
// while the MFMAs of slab k run, and one barrier per slab separates the two.  (Large
// launches use the software-pipelined form of this loop, see PIPE below.)
// A direct load writes 64 lanes x 16 bytes contiguously, i.e. 8 LDS rows of 128 bytes,
// so rows cannot be padded; bank conflicts of the fragment reads (32 rows, one 16-byte
// chunk each) are avoided by an XOR swizzle instead: logical chunk c of row r lives at
// chunk c ^ ((r >> 1) & 7).  The swizzle is applied on the global-address side of the
// load (lane l fetches the logical chunk that belongs at its fixed LDS position).
// Each 64-lane wave owns a (BM/WM) x (BN/WN) sub-tile built from 32x32x16 MFMAs.  The
// weights are fed as the MFMA "A" operand and the activations as "B", so a lane ends
// up holding 4 CONSECUTIVE output features of one row - the epilogue (bias, SiLU,
// gate*y + residual) then works on contiguous 8- or 16-byte pieces of row-major C.
// Workgroup ids are remapped so that the ids that land on one XCD (id mod 8) walk
// the N-tiles of the same rows of A: A is fetched from HBM once and the weight
// matrix sits in every XCD's L2.
// Requirements (checked by the launcher): K % 64 == 0, N % 64 == 0, 16-byte
// aligned A, B and leading dimensions; M is free (rows past M are clamped on load
// and never stored).
#include <cstdlib>
#include <type_traits>

#include "internal.hpp"

namespace csd {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

__device__ __forceinline__ float silu_fast(float a) { return a / (1.0f + __expf(-a)); }

struct Params {
    const bf16_t* A; int lda;
    const bf16_t* B;            // ldb = K
    const float* bias;
    void* C; int ldc;
    const bf16_t* gate; int ldg;
    int M, N, K;
    int tiles_m, tiles_n;
    int panel;                  // > 0: an XCD walks its tiles in column panels of this many N-tiles
    int ksplit;                 // length of the K range of one workgroup row (gridDim.y ranges; = K without split-K)
    long long c_split_stride;   // elements between the partial products of consecutive K ranges
    unsigned long long* ts;     // optional: [0] min start, [1] max end over the workgroups (profiling)
};

// s_waitcnt with only vmcnt set (expcnt and lgkmcnt left at "don't wait")
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// s_waitcnt with only lgkmcnt(0) set: this wave's LDS reads have returned
__device__ __forceinline__ void wait_lds_reads() { __builtin_amdgcn_s_waitcnt(0xC07F); }

template <int BM, int BN, int WM, int WN, int BK, int NST, int EPI, bool OUT_F32, bool PIPE = false>
__global__ __launch_bounds__(WM * WN * 64) void k_gemm_bf16(Params p) {
    constexpr int NW = WM * WN;
    constexpr bool WIDE_EPI = (NW == 4 && BM == 256);     // measured per tile form
    constexpr int TM = BM / WM, TN = BN / WN;          // per-wave tile
    constexpr int FM = TM / 32, FN = TN / 32;          // 32x32 blocks per wave
    constexpr int ROW_B = BK * 2;                      // bytes per LDS row
    constexpr int CPR = BK / 8;                        // 16-byte chunks per row (8 or 4)
    constexpr int RPL = 64 / CPR;                      // rows written by one wave-wide direct load
    constexpr int SH = (CPR == 8) ? 1 : 2;             // log2(rows per 256-byte bank window)
    constexpr int GROUPS = (BM + BN) / RPL;            // direct loads (1 KiB of LDS each) per slab
    constexpr int GPW = GROUPS / NW;                   // ... issued by each wave
    static_assert(BK == 64 || BK == 32, "BK");
    static_assert(GROUPS % NW == 0 && NW % 2 == 0 && (BM / RPL) % 2 == 0, "loader mapping");
    constexpr int STAGE_B = (BM + BN) * ROW_B;
    static_assert(NW * 32 * TN * 4 <= NST * STAGE_B, "epilogue staging must fit in the LDS of the main loop");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    if (p.ts && threadIdx.x == 0) atomicMin(p.ts, (unsigned long long)__builtin_amdgcn_s_memrealtime());

    // ---- tile of this workgroup: ids sharing id%8 (one XCD) sweep n first, then m
    int tm, tn;
    {
        int tile = blockIdx.x;
        const int total = p.tiles_m * p.tiles_n;
        const int per_xcd = total / 8;
        const bool by_xcd = per_xcd * 8 == total;
        if (by_xcd) tile = (tile % 8) * per_xcd + tile / 8;
        tm = tile / p.tiles_n; tn = tile % p.tiles_n;
        if (by_xcd && p.panel > 0 && per_xcd % p.tiles_n == 0) {
            // very wide N (the stacked modulation layers): the XCD's rows x panel of N-tiles at a
            // time, so that the weight panel in flight is shared by all its rows through L2 and
            // its few A row-tiles stay there from panel to panel
            const int rows = per_xcd / p.tiles_n, i = (int)blockIdx.x / 8;
            const int per_panel = p.panel * rows, pn = i / per_panel, j = i % per_panel;
            tm = ((int)blockIdx.x % 8) * rows + j / p.panel;
            tn = pn * p.panel + j % p.panel;
        }
    }
    const int64_t m0 = (int64_t)tm * BM;
    const int n0 = tn * BN;
    // split-K: workgroup row blockIdx.y sums its own K range into its own copy of C
    const bf16_t* const Ap = p.A + (size_t)blockIdx.y * p.ksplit;
    const bf16_t* const Bp = p.B + (size_t)blockIdx.y * p.ksplit;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, khalf = lane >> 5;

    // ---- loader: lane (lr, pc) of a direct load writes LDS row lr, physical chunk pc, and
    // fetches the logical chunk pc ^ swizzle(row) that belongs there
    const int lr = lane / CPR, pc = lane % CPR;
    const int ld_swz = (CPR == 8) ? ((((wave & 1) << 2) + (lr >> 1)) & 7) : ((lr >> 2) & 3);
    const int ld_chunk = pc ^ ld_swz;
    auto issue_loads_part = [&](int stage, int k0, int i0, int i1) {
#pragma unroll
        for (int i = i0; i < i1; ++i) {
            const int g = wave + i * NW;               // rows RPL*g .. RPL*g+RPL-1 of the slab
            const int row = g * RPL + lr;
            const bf16_t* src;
            if (g < BM / RPL) {                        // uniform per wave and i
                int64_t r = m0 + row;
                r = r < p.M ? r : (int64_t)p.M - 1;
                src = Ap + r * p.lda + k0 + ld_chunk * 8;
            } else {
                src = Bp + (size_t)(n0 + row - BM) * p.K + k0 + ld_chunk * 8;
            }
            __builtin_amdgcn_global_load_lds(src, (__attribute__((address_space(3))) void*)(smem + stage * STAGE_B + g * 1024),
                                             16, 0, 0);
        }
    };
    auto issue_loads = [&](int stage, int k0) { issue_loads_part(stage, k0, 0, GPW); };

    // ---- fragment read offsets (bytes) of this lane for the k16-steps of a slab
    const int swz = (l32 >> SH) & (CPR - 1);
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

    const int nk = p.ksplit / BK;
    if constexpr (PIPE) {
        // ---- software-pipelined main loop (two stages of 64, at least 4 slabs).  Fragments are
        // double-buffered in registers, so the LDS reads of k16-step kk+1 run under the MFMAs of
        // step kk.  The ONE barrier per slab sits between steps 2 and 3: by then every wave holds
        // the last fragments of slab s in registers, so the stage of slab s is free for slab s+2,
        // and slab s+1 (requested one slab earlier) has landed, so its first fragments are read
        // under the MFMAs of step 3 - no wave ever waits at a slab boundary with an empty MFMA
        // pipe.  The requests for slab s+2 go out in two halves, after the barrier and in step 0
        // of the next slab, so that no wave sits long in the queue of the load unit.
        static_assert(BK == 64 && NST == 2, "pipelined loop: two stages of 64");
        bf16x8 fa[2][FM], fb[2][FN];
        auto read_frags = [&](auto buf_c, int stage, int kk) {
            constexpr int buf = decltype(buf_c)::value;
            const unsigned char* sa = smem + stage * STAGE_B + a_row_off + koff[kk];
            const unsigned char* sb = smem + stage * STAGE_B + b_row_off + koff[kk];
#pragma unroll
            for (int i = 0; i < FM; ++i) fa[buf][i] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(sa + i * 32 * ROW_B));
#pragma unroll
            for (int j = 0; j < FN; ++j) fb[buf][j] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(sb + j * 32 * ROW_B));
        };
        // One k16-step in a pinned instruction order: behind each of the first FM+FN MFMAs
        // (operands from buffer CUR) one fragment read of the NEXT step (into the other
        // buffer), behind the last MFMAs the NL load requests [ld_i0, ld_i0+NL) of a later slab.
        // The scheduling barriers keep the compiler from clustering them again.
        auto step = [&](auto cur_c, auto read_c, int rd_stage, int rd_kk, auto nl_c, int ld_stage, int ld_k0, int ld_i0) {
            constexpr int CUR = decltype(cur_c)::value, NXT = CUR ^ 1, NL = decltype(nl_c)::value;
            constexpr bool READ = decltype(read_c)::value;
            constexpr int NM = FM * FN, NR = FM + FN;
            static_assert(NR <= NM && NL <= 2 * (NM - NR + 1), "step layout");
            const unsigned char* sa = smem + rd_stage * STAGE_B + a_row_off + koff[rd_kk];
            const unsigned char* sb = smem + rd_stage * STAGE_B + b_row_off + koff[rd_kk];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < NM; ++u) {
                const int i = u / FN, j = u % FN;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[CUR][j], fa[CUR][i], acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                if (READ && u < NR) {
                    // fb first: the first MFMA of the next step then needs only reads 0 .. FN
                    if (u < FN) fb[NXT][u] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(sb + u * 32 * ROW_B));
                    else fa[NXT][u - FN] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(sa + (u - FN) * 32 * ROW_B));
                    __builtin_amdgcn_sched_barrier(0);
                }
                // load requests ride behind the MFMAs from index NR-1 on, two at a time
                if (NL > 0 && u >= NR - 1) {
                    const int l0 = (u - (NR - 1)) * 2;
                    if (l0 < NL) {
                        issue_loads_part(ld_stage, ld_k0, ld_i0 + l0, ld_i0 + (l0 + 2 < NL ? l0 + 2 : NL));
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        };
        typedef std::integral_constant<int, 0> I0;
        typedef std::integral_constant<int, 1> I1;
        constexpr int H1 = (GPW + 1) / 2, H2 = GPW - H1;      // the two halves of a slab's load requests
        typedef std::integral_constant<int, H1> IH1;
        typedef std::integral_constant<int, H2> IH2;
        typedef std::true_type RD;
        auto slab = [&](auto first_c, auto next1_c, auto next2_c, int s) {
            constexpr bool FIRST = decltype(first_c)::value, NEXT1 = decltype(next1_c)::value, NEXT2 = decltype(next2_c)::value;
            const int st = s & 1;
            if constexpr (!FIRST && NEXT1) step(I0{}, RD{}, st, 1, IH2{}, st ^ 1, (s + 1) * BK, H1);
            else step(I0{}, RD{}, st, 1, I0{}, 0, 0, 0);
            step(I1{}, RD{}, st, 2, I0{}, 0, 0, 0);
            step(I0{}, RD{}, st, 3, I0{}, 0, 0, 0);
            if constexpr (NEXT1) wait_vmcnt<0>();
            wait_lds_reads();
            __builtin_amdgcn_s_barrier();
            if constexpr (NEXT2) step(I1{}, RD{}, st ^ 1, 0, IH1{}, st, (s + 2) * BK, 0);
            else if constexpr (NEXT1) step(I1{}, RD{}, st ^ 1, 0, I0{}, 0, 0, 0);
            else step(I1{}, std::false_type{}, 0, 0, I0{}, 0, 0, 0);
        };
        issue_loads(0, 0);
        issue_loads(1, BK);
        wait_vmcnt<GPW>();
        __builtin_amdgcn_s_barrier();
        read_frags(I0{}, 0, 0);
        slab(std::true_type{}, std::true_type{}, std::true_type{}, 0);
        for (int s = 1; s < nk - 2; ++s) slab(std::false_type{}, std::true_type{}, std::true_type{}, s);
        slab(std::false_type{}, std::true_type{}, std::false_type{}, nk - 2);
        slab(std::false_type{}, std::false_type{}, std::false_type{}, nk - 1);
    } else {
    // ---- main loop: NST-deep ring of slabs.  At step kt the slabs kt .. kt+NST-2 are in
    // flight; wait for slab kt only, barrier (which also says everyone is done reading
    // slab kt-1), refill the stage of slab kt-1 with slab kt+NST-1, then compute slab kt.
#pragma unroll
    for (int s = 0; s < NST - 1; ++s)
        if (s < nk) issue_loads(s, s * BK);
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + NST - 2 < nk) wait_vmcnt<GPW * (NST - 2)>(); else wait_vmcnt<0>();
        __syncthreads();
        if (kt + NST - 1 < nk) issue_loads((kt + NST - 1) % NST, (kt + NST - 1) * BK);
        const unsigned char* sa = smem + (kt % NST) * STAGE_B + a_row_off;
        const unsigned char* sb = smem + (kt % NST) * STAGE_B + b_row_off;
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
    }
    }
    __syncthreads();      // all waves are done with the last slab: LDS is free for the epilogue

    // ---- epilogue.  After the MFMAs a lane holds, per 32x32 block (i,j) and q, 4
    // consecutive features of ONE row, i.e. a wave store would touch 32 rows with 16
    // bytes each.  Each wave therefore transposes one 32-row slab at a time through a
    // private piece of the (now idle) LDS and walks it row-wise: NCH lanes cover the
    // TN*4 contiguous bytes of a row, so global loads and stores use whole cache lines.
    constexpr int NCH = TN / 4;                              // 16-byte chunks per staged row
    constexpr int LPR = (64 % NCH == 0) ? NCH : 32;          // lanes per row (TN = 96: 24 of 32 lanes work)
    constexpr int RPP = 64 / LPR;                            // rows per pass of the wave
    static_assert(NCH <= LPR && (NCH % 8 == 0), "epilogue row mapping");
    float* stg = reinterpret_cast<float*>(smem + wave * (32 * TN * 4));
    // the XOR must map [0,NCH) onto itself: within aligned groups of 16 (NCH a multiple of 16) or 8
    auto stg_swz = [](int row) { return NCH % 16 == 0 ? (row & 15) : (NCH == 8 ? ((row >> 1) & 7) : (row & 7)); };
    const int rd_row0 = lane / LPR, rd_c = lane % LPR;
    // The bias is fetched and WAITED FOR here, in code every lane runs.  If its first use
    // sat in the row-guarded blocks below, the compiler could not tell at the next block
    // whether the wait had happened and would wait for "all memory operations" again in
    // every pass, which also waits for the previous pass's store: the passes would run
    // one store round trip at a time.
    const int n_ep = n0 + wn * TN + (rd_c < NCH ? rd_c : 0) * 4;
    float4 bb = make_float4(0.f, 0.f, 0.f, 0.f);
    auto load_bb = [&]() {
        bb = *reinterpret_cast<const float4*>(p.bias + n_ep);
        if (blockIdx.y != 0) bb = make_float4(0.f, 0.f, 0.f, 0.f);   // the bias goes into the first K range only
        asm volatile("" : "+v"(bb.x), "+v"(bb.y), "+v"(bb.z), "+v"(bb.w));
    };
    // Tiles that lie wholly inside M take the copy of the code without row guards, where the
    // compiler is free to batch the LDS reads and stores of a slab.
    auto emit = [&](auto guard_c) {
        constexpr bool GUARD = decltype(guard_c)::value;
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int c = j * 8 + q * 2 + khalf;
                    *reinterpret_cast<float4*>(stg + l32 * TN + ((c ^ stg_swz(l32)) << 2)) =
                        make_float4(acc[i][j][4 * q + 0], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                }
            if (rd_c >= NCH) continue;                           // idle lanes of a row (uniform over i)
            const int n = n_ep;
#pragma unroll
            for (int pass = 0; pass < 32 / RPP; ++pass) {
                const int row = pass * RPP + rd_row0;
                const float4 a4 = *reinterpret_cast<const float4*>(stg + row * TN + ((rd_c ^ stg_swz(row)) << 2));
                const int64_t m = m0 + wm * TM + i * 32 + row;
                if (GUARD && m >= p.M) continue;
                float v0 = a4.x + bb.x, v1 = a4.y + bb.y, v2 = a4.z + bb.z, v3 = a4.w + bb.w;
                if (EPI == EPI_BIAS_SILU) { v0 = silu_fast(v0); v1 = silu_fast(v1); v2 = silu_fast(v2); v3 = silu_fast(v3); }
                if (EPI == EPI_GATE_RES) {
                    const uint2 g = *reinterpret_cast<const uint2*>(p.gate + m * p.ldg + n);
                    float* cp = (float*)p.C + m * p.ldc + n;
                    const float4 c = *reinterpret_cast<const float4*>(cp);
                    v0 = fmaf(bf16_to_f32((bf16_t)(g.x & 0xFFFF)), v0, c.x);
                    v1 = fmaf(bf16_to_f32((bf16_t)(g.x >> 16)), v1, c.y);
                    v2 = fmaf(bf16_to_f32((bf16_t)(g.y & 0xFFFF)), v2, c.z);
                    v3 = fmaf(bf16_to_f32((bf16_t)(g.y >> 16)), v3, c.w);
                    *reinterpret_cast<float4*>(cp) = make_float4(v0, v1, v2, v3);
                } else if (OUT_F32) {
                    *reinterpret_cast<float4*>((float*)p.C + (size_t)blockIdx.y * p.c_split_stride + m * p.ldc + n) = make_float4(v0, v1, v2, v3);
                } else {
                    *reinterpret_cast<uint2*>((bf16_t*)p.C + m * p.ldc + n) =
                        make_uint2(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3));
                }
            }
        }
    };
    // bf16 output (plain or SiLU epilogue) with an even number of chunks per row: the same staging, but a
    // lane takes two neighbouring chunks and stores 16 bytes (8 features), half as many store instructions
    auto emit_wide = [&](auto guard_c) {
        constexpr bool GUARD = decltype(guard_c)::value;
        constexpr int LPR2 = LPR / 2, RPP2 = 64 / LPR2, NCH2 = NCH / 2;
        const int row0 = lane / LPR2, c2 = lane % LPR2;
        const int n8 = n0 + wn * TN + (c2 < NCH2 ? c2 : 0) * 8;
        float4 b0 = *reinterpret_cast<const float4*>(p.bias + n8), b1 = *reinterpret_cast<const float4*>(p.bias + n8 + 4);
        asm volatile("" : "+v"(b0.x), "+v"(b0.y), "+v"(b0.z), "+v"(b0.w), "+v"(b1.x), "+v"(b1.y), "+v"(b1.z), "+v"(b1.w));
#pragma unroll
        for (int i = 0; i < FM; ++i) {
#pragma unroll
            for (int j = 0; j < FN; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int c = j * 8 + q * 2 + khalf;
                    *reinterpret_cast<float4*>(stg + l32 * TN + ((c ^ stg_swz(l32)) << 2)) =
                        make_float4(acc[i][j][4 * q + 0], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                }
            if (c2 >= NCH2) continue;
#pragma unroll
            for (int pass = 0; pass < 32 / RPP2; ++pass) {
                const int row = pass * RPP2 + row0;
                const float4 a0 = *reinterpret_cast<const float4*>(stg + row * TN + (((2 * c2) ^ stg_swz(row)) << 2));
                const float4 a1 = *reinterpret_cast<const float4*>(stg + row * TN + (((2 * c2 + 1) ^ stg_swz(row)) << 2));
                const int64_t m = m0 + wm * TM + i * 32 + row;
                if (GUARD && m >= p.M) continue;
                float v0 = a0.x + b0.x, v1 = a0.y + b0.y, v2 = a0.z + b0.z, v3 = a0.w + b0.w;
                float v4 = a1.x + b1.x, v5 = a1.y + b1.y, v6 = a1.z + b1.z, v7 = a1.w + b1.w;
                if (EPI == EPI_BIAS_SILU) {
                    v0 = silu_fast(v0); v1 = silu_fast(v1); v2 = silu_fast(v2); v3 = silu_fast(v3);
                    v4 = silu_fast(v4); v5 = silu_fast(v5); v6 = silu_fast(v6); v7 = silu_fast(v7);
                }
                *reinterpret_cast<uint4*>((bf16_t*)p.C + m * p.ldc + n8) =
                    make_uint4(pack_bf16x2(v0, v1), pack_bf16x2(v2, v3), pack_bf16x2(v4, v5), pack_bf16x2(v6, v7));
            }
        }
    };
    if constexpr (!OUT_F32 && EPI != EPI_GATE_RES && NCH % 2 == 0 && LPR % 2 == 0 && WIDE_EPI) {
        // (the launcher sends bf16 outputs whose rows do not start on 16-byte boundaries to another tile form)
        if (m0 + BM <= p.M) emit_wide(std::false_type{}); else emit_wide(std::true_type{});
    } else {
        load_bb();
        if (m0 + BM <= p.M) emit(std::false_type{}); else emit(std::true_type{});
    }
    if (p.ts && (threadIdx.x & 63) == 0) atomicMax(p.ts + 1, (unsigned long long)__builtin_amdgcn_s_memrealtime());
}

template <int BM, int BN, int WM, int WN, int BK, int NST, bool PIPE = false>
hipError_t launch_cfg(const GemmArgs& g, hipStream_t st) {
    Params p;
    p.A = (const bf16_t*)g.A; p.lda = g.lda; p.B = (const bf16_t*)g.B; p.bias = g.bias;
    p.C = g.C; p.ldc = g.ldc; p.gate = (const bf16_t*)g.gate; p.ldg = g.ldg;
    p.M = g.M; p.N = g.N; p.K = g.K; p.ts = g.ts;
    const int splits = g.k_splits > 1 ? g.k_splits : 1;
    // split-K: fp32 partial products only (plain bias epilogue), each range a whole number of slabs
    if (splits > 1 && (g.epi != EPI_BIAS || !g.c_is_f32 || g.K % (splits * BK) != 0 || PIPE)) return hipErrorInvalidValue;
    p.ksplit = g.K / splits; p.c_split_stride = g.c_split_stride;
    p.tiles_m = (g.M + BM - 1) / BM; p.tiles_n = g.N / BN;
    p.panel = 0;
    if (p.tiles_n > 16)
        for (int d = 16; d >= 8; --d)
            if (p.tiles_n % d == 0) { p.panel = d; break; }
    const size_t smem = (size_t)NST * (BM + BN) * BK * 2;
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), (unsigned)splits), block(WM * WN * 64);
#define CSD_LAUNCH(EPI, F32)                                                                                   \
    do {                                                                                                       \
        auto kern = k_gemm_bf16<BM, BN, WM, WN, BK, NST, EPI, F32, PIPE>;                                            \
        static bool attr_done = false;                                                                          \
        if (!attr_done) {                                                                                       \
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem); \
            if (e != hipSuccess) return e;                                                                      \
            attr_done = true;                                                                                   \
        }                                                                                                       \
        hipLaunchKernelGGL(kern, grid, block, smem, st, p);                                                     \
    } while (0)
    switch (g.epi) {
        case EPI_BIAS: if (g.c_is_f32) CSD_LAUNCH(EPI_BIAS, true); else CSD_LAUNCH(EPI_BIAS, false); break;
        case EPI_BIAS_SILU: if (g.c_is_f32) CSD_LAUNCH(EPI_BIAS_SILU, true); else CSD_LAUNCH(EPI_BIAS_SILU, false); break;
        case EPI_GATE_RES: CSD_LAUNCH(EPI_GATE_RES, true); break;
        default: return hipErrorInvalidValue;
    }
#undef CSD_LAUNCH
    return hipGetLastError();
}

// tuning hook: environment variable CSD_GEMM_VARIANT forces a tile shape / main loop (see launch_gemm_bf16)
int gemm_variant_override() {
    static int v = -2;
    if (v == -2) { const char* e = getenv("CSD_GEMM_VARIANT"); v = (e && *e) ? atoi(e) : -1; }
    return v;
}

}  // namespace

hipError_t launch_gemm_bf16(const GemmArgs& g, hipStream_t st) {
    if (g.M == 0) return hipSuccess;
    if (g.K % 64 != 0 || g.N % 64 != 0 || g.lda % 8 != 0 || g.ldc % 4 != 0) return hipErrorInvalidValue;
    if (((uintptr_t)g.A & 15u) || ((uintptr_t)g.B & 15u) || ((uintptr_t)g.C & 15u)) return hipErrorInvalidValue;
    if (g.epi == EPI_GATE_RES && (g.ldg % 4 != 0 || ((uintptr_t)g.gate & 7u))) return hipErrorInvalidValue;
    // Tile shapes (CSD_GEMM_VARIANT forces one where it fits, a tuning hook):
    //   12 256x256, 4 waves of 128x128 (one per SIMD, the 256 accumulators of a lane in the accumulation
    //      registers), software-pipelined main loop - every large launch.  Alone on the chip it is 3 %
    //      behind the 8-wave form below (the same 1.5 us per slab, a slower epilogue), but the whole path
    //      gains 1-2 % on every workload: it reads a third fewer fragments from LDS per MFMA and leaves
    //      a quarter of each SIMD's registers to the row kernels of the other chains on the same CU.
    //   9  the same tile as 8 waves of 128x64
    //   1  the same tile with the plain two-stage loop (also serves K < 256)
    //   8  256x192, 8 waves of 64x96: large launches whose N only 192 divides.  (Alone on the chip it
    //      also wins where both divide, e.g. N = 2304: 949 against 878 TFLOP/s, but it moves 17 % more
    //      bytes from L2 per flop and loses on the whole path, where several chains share the chip.)
    //   3  64x64, 4 waves: below 2048 rows a launch is latency-bound and wants many small workgroups
    //      (one head pass at 256 / 1024 rows: 263 / 290 us against 343 / 366 with 128x128 tiles; a
    //      deeper ring of slabs buys nothing there)
    int variant = gemm_variant_override();
    if (variant != 1 && variant != 3 && variant != 8 && variant != 9 && variant != 12) {
        if (g.M >= 2048 && g.N % 256 == 0) variant = 12;
        else if (g.M >= 2048 && g.N % 192 == 0) variant = 8;
        else variant = 3;
    }
    if (g.k_splits > 1) variant = 3;
    if (variant == 12 && !g.c_is_f32 && g.epi != EPI_GATE_RES && g.ldc % 8 != 0) variant = 9;   // 16-byte stores of the 4-wave form
    if ((variant == 1 || variant == 9 || variant == 12) && g.N % 256 != 0) variant = (g.N % 192 == 0) ? 8 : 3;
    if (variant == 8 && g.N % 192 != 0) variant = 3;
    switch (variant) {
        case 1: return launch_cfg<256, 256, 2, 4, 64, 2>(g, st);
        case 9: if (g.K >= 256) return launch_cfg<256, 256, 2, 4, 64, 2, true>(g, st);
                return launch_cfg<256, 256, 2, 4, 64, 2>(g, st);
        case 12: if (g.K >= 256) return launch_cfg<256, 256, 2, 2, 64, 2, true>(g, st);
                 return launch_cfg<256, 256, 2, 4, 64, 2>(g, st);
        case 8: if (g.K >= 256) return launch_cfg<256, 192, 4, 2, 64, 2, true>(g, st);
                return launch_cfg<256, 192, 4, 2, 64, 2>(g, st);
        default: return launch_cfg<64, 64, 2, 2, 64, 2>(g, st);
    }
}

}  // namespace csd
