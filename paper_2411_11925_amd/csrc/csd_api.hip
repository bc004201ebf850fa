// C ABI of libcsd: argument checking, head set-up, and the host-side sequencing of
// the kernels of one lockstep denoising call.  See include/csd.h for the contract.
#include <cmath>
#include <cstdio>
#include <cstdarg>
#include <cstring>
#include <cstdlib>
#include <new>
#include <string>

#include "internal.hpp"

using namespace csd;

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap; va_start(ap, fmt); vsnprintf(buf, sizeof buf, fmt, ap); va_end(ap);
    g_err = buf;
    return code;
}

#define HIP_TRY(expr)                                                                         \
    do { hipError_t e_ = (expr);                                                              \
         if (e_ != hipSuccess) return fail(CSD_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

bool cfg_ok(const csd_head_cfg_t* c, const char** why) {
    if (!c) { *why = "cfg is NULL"; return false; }
    if (!(c->token_dim == 4 || c->token_dim == 8 || c->token_dim == 16)) { *why = "token_dim must be 4, 8 or 16"; return false; }
    if (c->width < 64 || c->width > 4096 || c->width % 64) { *why = "width must be a multiple of 64 in [64,4096]"; return false; }
    if (c->cond_dim < 8 || c->cond_dim > 16384 || c->cond_dim % 8) { *why = "cond_dim must be a multiple of 8 in [8,16384]"; return false; }
    if (c->n_blocks < 1 || c->n_blocks > 64) { *why = "n_blocks must be in [1,64]"; return false; }
    if (c->n_steps < 1 || c->n_steps > 4096) { *why = "n_steps must be in [1,4096]"; return false; }
    if (c->gemm_dtype != CSD_F32 && c->gemm_dtype != CSD_BF16) { *why = "gemm_dtype must be CSD_F32 or CSD_BF16"; return false; }
    if (c->schedule != CSD_COSINE && c->schedule != CSD_TABLE) { *why = "schedule must be CSD_COSINE or CSD_TABLE"; return false; }
    if (c->schedule == CSD_TABLE && !c->alpha_bar) { *why = "CSD_TABLE needs alpha_bar"; return false; }
    if (c->sampler != CSD_SAMPLER_DDPM && c->sampler != CSD_SAMPLER_DDIM) { *why = "sampler must be CSD_SAMPLER_DDPM or CSD_SAMPLER_DDIM"; return false; }
    if (c->sampler == CSD_SAMPLER_DDPM && c->ddim_eta != 0.f) { *why = "ddim_eta must be 0 with CSD_SAMPLER_DDPM"; return false; }
    if (c->sampler == CSD_SAMPLER_DDIM && !(c->ddim_eta > 0.f && c->ddim_eta <= 16.f)) { *why = "ddim_eta must be in (0,16]"; return false; }
    if (!(c->eps_skip_gain == c->eps_skip_gain)) { *why = "eps_skip_gain is NaN"; return false; }
    return true;
}

size_t param_count(const csd_head_cfg_t* c) {
    const size_t D = c->token_dim, C = c->cond_dim, W = c->width, L = c->n_blocks;
    size_t n = W * CSD_TIME_FEATURES + W + W * W + W + W * C + W + W * D + W;
    n += L * (3 * W * W + 3 * W + 2 * (W * W + W));
    n += 2 * W * W + 2 * W + 2 * D * W + 2 * D;
    return n;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// device buffers of one head for R rows, carved from the caller's workspace.  s, mod and fm do
// not depend on the trajectory (only on the step and the conditioning vector), so they are
// computed for `tb` consecutive denoising steps at once: [tb, R, .].  With few rows that turns
// the largest GEMMs of a step, which would be launch- and latency-bound at M = R, into GEMMs
// over tb*R rows; with many rows tb is 1.
struct HeadWs {
    float* e; void* s; void* mod; float* fm; float* h; void* u; void* a; void* y; float* o; float* x; float* acc;
    int tb;
};

constexpr size_t BATCH_BUDGET = (size_t)256 << 20;     // bytes of s + mod + fm a batch of steps may take

size_t batched_bytes_per_row(const csd_head* hd) {
    const size_t W = hd->W, act = hd->cfg.gemm_dtype == CSD_BF16 ? 2 : 4;
    return W * act + 3 * W * hd->L * act + 2 * W * 4;
}

// steps per batch for a call of R rows (row chunks of the call use the same value)
int steps_per_batch(const csd_head* hd, int64_t R) {
    if (R <= 0) return 1;
    const size_t per_step = (size_t)R * hd->reps * batched_bytes_per_row(hd);
    size_t tb = BATCH_BUDGET / per_step;
    if (tb < 1) tb = 1;
    if (tb > (size_t)hd->T) tb = (size_t)hd->T;
    return (int)tb;
}

// (R = trajectory rows; the head's activations have R * reps rows: 2 per row with guidance)
size_t head_ws_bytes(const csd_head* hd, int64_t R, int tb) {
    const size_t r = (size_t)R * hd->reps, W = hd->W, act = hd->cfg.gemm_dtype == CSD_BF16 ? 2 : 4;
    size_t n = 0;
    n += align_up(r * W * 4, 256);          // e
    n += align_up(tb * r * W * act, 256);   // s
    n += align_up(tb * r * 3 * W * hd->L * act, 256);  // mod: (shift, scale, gate) of all L blocks, [tb, R, L*3W]
    n += align_up(tb * r * 2 * W * 4, 256); // fm (fp32 in both modes)
    n += align_up(r * W * 4, 256);          // h
    n += align_up(r * W * 4, 256);          // u (fp32, bf16, or the [hi|lo] bf16 pair of the last layer)
    n += 2 * align_up(r * W * act, 256);    // a, y
    n += align_up(r * 64 * 4 * hd->out_splits, 256);   // o (output projection, padded to 64 columns; split-K partials)
    n += align_up((size_t)R * hd->D * 4, 256);      // x
    n += align_up((size_t)R * 4, 256);              // acc
    return n;
}

char* carve(const csd_head* hd, int64_t R, int tb, char* p, HeadWs* ws) {
    const size_t r = (size_t)R * hd->reps, W = hd->W, act = hd->cfg.gemm_dtype == CSD_BF16 ? 2 : 4;
    auto take = [&](size_t bytes) { char* q = p; p += align_up(bytes, 256); return q; };
    ws->tb = tb;
    ws->e = (float*)take(r * W * 4);
    ws->s = take(tb * r * W * act);
    ws->mod = take(tb * r * 3 * W * hd->L * act);
    ws->fm = (float*)take(tb * r * 2 * W * 4);
    ws->h = (float*)take(r * W * 4);
    ws->u = take(r * W * 4);
    ws->a = take(r * W * act);
    ws->y = take(r * W * act);
    ws->o = (float*)take(r * 64 * 4 * hd->out_splits);
    ws->x = (float*)take((size_t)R * hd->D * 4);
    ws->acc = (float*)take((size_t)R * 4);
    return p;
}

hipError_t gemm(const csd_head* hd, GemmArgs g, hipStream_t st) {
    return hd->cfg.gemm_dtype == CSD_BF16 ? launch_gemm_bf16(g, st) : launch_gemm_f32(g, st);
}

// optional timing of the dominant kernel (csd_profile_*): a hipEvent bracket on its launch stream,
// and (bf16 kernels) the span from the first workgroup's start to the last one's end on the device
struct Profile {
    std::vector<hipEvent_t> ev;     // 2 per launch
    std::vector<double> flops;
    unsigned long long* d_pair = nullptr;    // [max][2] device: start preset to ~0, end to 0
    size_t used = 0;                // launches recorded
    bool on = false;
} g_prof;

hipError_t gemm_timed(const csd_head* hd, const GemmArgs& g_in, hipStream_t st) {
    if (!g_prof.on || g_prof.used * 2 + 2 > g_prof.ev.size()) return gemm(hd, g_in, st);
    const size_t i = g_prof.used;
    GemmArgs g = g_in;
    g.ts = g_prof.d_pair ? g_prof.d_pair + 2 * i : nullptr;
    hipError_t e = hipEventRecord(g_prof.ev[2 * i], st);
    if (e != hipSuccess) return e;
    if ((e = gemm(hd, g, st)) != hipSuccess) return e;
    if ((e = hipEventRecord(g_prof.ev[2 * i + 1], st)) != hipSuccess) return e;
    g_prof.flops.push_back(2.0 * g.M * g.N * g.K);
    g_prof.used = i + 1;
    return hipSuccess;
}

// e = W_c z + b_c (once per call; fp32 in both modes)
hipError_t cond_embed(const csd_head* hd, const float* z, const HeadWs& ws, int64_t R, hipStream_t st) {
    GemmArgs g{};
    g.A = z; g.lda = hd->C; g.B = hd->cond.w; g.bias = hd->cond.b; g.C = ws.e; g.ldc = hd->W;
    g.M = (int)R; g.N = hd->W; g.K = hd->C; g.epi = EPI_BIAS; g.c_is_f32 = 1;
    return launch_gemm_f32(g, st);
}

// Before the first step of a batch: for the nb steps t_first, t_first-1, ..: s = SiLU(E_t + e),
// the (shift, scale, gate) of all L blocks - [nb*R, W] x [W, L*3W], one GEMM - and the final
// modulation (fp32, because it feeds eps_hat directly).
hipError_t batch_stage(const csd_head* hd, const HeadWs& ws, int t_first, int nb, int64_t R, hipStream_t st) {
    const int W = hd->W;
    const bool b16 = hd->cfg.gemm_dtype == CSD_BF16;
    hipError_t e = launch_cond_silu(ws.e, hd->d_time_emb + (size_t)t_first * W, nb, ws.s, b16 ? ACT_BF16 : ACT_F32, R, W, st);
    if (e != hipSuccess) return e;
    GemmArgs g{};
    g.M = (int)(R * nb); g.K = W; g.lda = W; g.A = ws.s; g.epi = EPI_BIAS;
    g.B = b16 ? (const void*)hd->mod_all.w16 : (const void*)hd->mod_all.w; g.bias = hd->mod_all.b;
    g.C = ws.mod; g.N = hd->mod_all.n_out; g.ldc = g.N; g.c_is_f32 = 0;
    if ((e = gemm_timed(hd, g, st)) != hipSuccess) return e;
    g.B = b16 ? (const void*)hd->fmod.w16 : (const void*)hd->fmod.w; g.bias = hd->fmod.b;
    g.C = ws.fm; g.N = hd->fmod.n_out; g.ldc = g.N; g.c_is_f32 = 1;
    return gemm(hd, g, st);
}

// The trajectory-dependent part of one denoising step, in phases p = 0 .. L+1:
//   p = 0:       block_pre(first)
//   1 <= p <= L: fc1_{p-1}, fc2_{p-1}, then block_pre(middle; final for p = L)
//   p = L+1:     output projection (the transition follows, by the caller)
// k = index of the step within its batch (selects the slice of s / mod / fm).
hipError_t phase_gemm(const csd_head* hd, const HeadWs& ws, int p, int64_t R, hipStream_t sg) {
    const int W = hd->W, L = hd->L;
    const bool b16 = hd->cfg.gemm_dtype == CSD_BF16;
    hipError_t e;
    GemmArgs g{};
    g.M = (int)R; g.K = W; g.lda = W;
    if (p == L + 1) {
        // o = Lin_out(u), padded to 64 columns.  In bf16 mode u is the [hi | lo] pair against [w | w].
        g.N = 64; g.K = b16 ? 2 * W : W; g.A = ws.u; g.lda = g.K;
        g.B = b16 ? (const void*)hd->out_pad.w16 : (const void*)hd->out_pad.w; g.bias = hd->out_pad.b;
        g.C = ws.o; g.ldc = 64; g.epi = EPI_BIAS; g.c_is_f32 = 1;
        // a 64-column output has few tiles and a long K: cut K so that the launch is not one long
        // dependent chain per workgroup; the transition adds the partial products
        g.k_splits = hd->out_splits; g.c_split_stride = (int64_t)R * 64;
        return gemm(hd, g, sg);
    }
    if (p >= 1) {
        const int l = p - 1;           // a = silu(fc1 u);  y = fc2 a
        g.A = ws.u; g.B = b16 ? (const void*)hd->fc1[l].w16 : (const void*)hd->fc1[l].w;
        g.bias = hd->fc1[l].b; g.C = ws.a; g.ldc = W; g.N = W; g.epi = EPI_BIAS_SILU; g.c_is_f32 = 0;
        if ((e = gemm(hd, g, sg)) != hipSuccess) return e;
        g.A = ws.a; g.B = b16 ? (const void*)hd->fc2[l].w16 : (const void*)hd->fc2[l].w;
        g.bias = hd->fc2[l].b; g.C = ws.y; g.epi = EPI_BIAS;
        if ((e = gemm(hd, g, sg)) != hipSuccess) return e;
    }
    return hipSuccess;
}

// elementwise part of phases 0..L (residual or input projection, LN, modulation -> u)
hipError_t phase_elem(const csd_head* hd, const HeadWs& ws, int p, int k, int64_t R, hipStream_t se) {
    const int W = hd->W, L = hd->L;
    const bool b16 = hd->cfg.gemm_dtype == CSD_BF16;
    const size_t asz = b16 ? 2 : 4;
    BlockPreArgs bp{};
    bp.act = b16 ? ACT_BF16 : ACT_F32; bp.h = ws.h; bp.y = ws.y; bp.u = ws.u; bp.ln_eps = hd->ln_eps;
    bp.R = R; bp.W = W; bp.D = hd->D;
    bp.x = ws.x; bp.x_div = hd->reps; bp.w_in = hd->in.w; bp.b_in = hd->in.b; bp.w_in_t = hd->d_in_t;
    bp.mode = (p == 0) ? 0 : (p == L ? 2 : 1);
    const int ld_all = 3 * W * L;          // block l's (shift, scale, gate) sit at columns [l*3W, (l+1)*3W) of a mod row
    const char* mod_k = (const char*)ws.mod + (size_t)k * R * ld_all * asz;        // step k of the batch
    bp.mod = (p == L) ? (const void*)(ws.fm + (size_t)k * R * 2 * W) : (const void*)(mod_k + (size_t)p * 3 * W * asz);
    bp.ldm = (p == L) ? 2 * W : ld_all;
    if (p > 0) { bp.gate = mod_k + ((size_t)(p - 1) * 3 * W + 2 * W) * asz; bp.ldg = ld_all; }
    return launch_block_pre(bp, se);
}

// the trajectory-dependent part of a step on one stream
hipError_t head_body(const csd_head* hd, const HeadWs& ws, int k, int64_t R, hipStream_t st) {
    hipError_t e;
    for (int p = 0; p <= hd->L + 1; ++p) {
        if ((e = phase_gemm(hd, ws, p, R, st)) != hipSuccess) return e;
        if (p <= hd->L && (e = phase_elem(hd, ws, p, k, R, st)) != hipSuccess) return e;
    }
    return hipSuccess;
}

TransArgs trans_args(const csd_head* hd, const HeadWs& ws, int t, int64_t R) {
    TransArgs f{};
    f.o = ws.o; f.ldo = 64; f.R = R; f.D = hd->D; f.x = ws.x; f.acc = ws.acc;
    f.o_splits = hd->out_splits; f.o_split_stride = (int64_t)R * hd->reps * 64;
    f.coef = hd->coef[t]; f.t = t;
    f.row_stride = 1; f.row_shift = 0; f.rng_stream = CSD_STREAM_TRAJ;
    f.reps = hd->reps; f.cfg_scale = hd->cfg_scale;
    return f;
}

// Side streams (default priority) with their fork/join events, one set per device, created
// on first use and kept until the process ends.  CSD_SINGLE_STREAM=1 keeps everything on
// the caller's stream; CSD_ROW_CHUNKS=n (1..4) sets how many row chunks run as separate chains.
constexpr int MAX_SIDE = 7;
struct SideStreams {
    hipStream_t stream[MAX_SIDE + 1] = {};
    hipEvent_t join[MAX_SIDE + 1] = {};
    hipEvent_t fork = nullptr;
    bool ok = false;
};

SideStreams* side_streams(int device) {
    static SideStreams sets[16];
    static int disabled = -1;
    if (disabled < 0) { const char* e = getenv("CSD_SINGLE_STREAM"); disabled = (e && *e == '1') ? 1 : 0; }
    if (disabled || device < 0 || device >= 16) return nullptr;
    SideStreams& s = sets[device];
    if (!s.ok) {
        if (hipEventCreateWithFlags(&s.fork, hipEventDisableTiming) != hipSuccess) return nullptr;
        for (int i = 0; i <= MAX_SIDE; ++i) {
            if (hipStreamCreateWithFlags(&s.stream[i], hipStreamNonBlocking) != hipSuccess) return nullptr;
            if (hipEventCreateWithFlags(&s.join[i], hipEventDisableTiming) != hipSuccess) return nullptr;
        }
        s.ok = true;
    }
    return &s;
}

int row_chunks_setting() {
    static int v = -1;
    if (v < 0) { const char* e = getenv("CSD_ROW_CHUNKS"); v = (e && *e) ? atoi(e) : 0; if (v < 0 || v > 4) v = 0; }
    return v;
}

struct DeviceGuard {
    int prev = -1; bool ok = false;
    explicit DeviceGuard(int dev) { if (hipGetDevice(&prev) == hipSuccess && hipSetDevice(dev) == hipSuccess) ok = true; }
    ~DeviceGuard() { if (prev >= 0) (void)hipSetDevice(prev); }
};


// One chain = one head walking rows [0, n) of its slice from x_T to x_0 on its own stream.
// Row r of the chain is row r*row_stride + row_shift of the slice's summary and, behind
// row_offset, of the noise counters.
struct Chain {
    const csd_head* hd; HeadWs ws; const float* z; int64_t n;
    uint64_t row_offset; int64_t row_stride, row_shift; int rng_stream;
    float* summary; int is_target; float* tokens;
    // path-ratio comparison (all zero in the method's own path): how acc is formed, the stored
    // path [T+1][path_stride] floats (slot t holds x_t of this chain's rows) that the chain
    // writes (path_write) or follows, whether acc starts at 1/2 ||x_T||^2, the own final sample
    int path_mode; float* path; int64_t path_stride; int path_write; int init_norm; float* x0_own;
    hipStream_t s;
};

// Cuts n rows into row chunks (multiples of 256 rows, so every result is bit-identical to a
// single-chain run): 2 for >= 8192 rows unless CSD_ROW_CHUNKS says otherwise.
int plan_chunks(int64_t n, bool have_side, int64_t* chunk_rows) {
    int n_chunks = row_chunks_setting();
    if (n_chunks == 0) n_chunks = (n >= 8192) ? 2 : 1;
    if (!have_side) n_chunks = 1;
    int64_t rows = ((n + n_chunks - 1) / n_chunks + 255) / 256 * 256;
    if (rows >= n) { n_chunks = 1; rows = n; }
    *chunk_rows = rows;
    return (int)((n + rows - 1) / rows);
}

// Runs the chains to the end.  Chain 0 uses the caller's stream, the others side streams of
// default priority; fork and join are events on the caller's stream, the host is never
// synchronised.  The chains run free: one chain's memory-bound kernels and GEMM epilogues fill
// the gaps of another chain's MFMA loops.  (Tying them into a fixed GEMM/row-kernel pipeline
// with events was measured and is slower: every cross-stream hand-over costs more than the
// overlap it buys.  The same holds for running the trajectory-independent part of step t-1 on a
// second stream beside step t: 265 against 252 ms per step.)
int run_chains(Chain* chains, int n_chains, uint64_t seed, float tau, hipStream_t st, SideStreams* side) {
    for (int i = 0; i < n_chains; ++i) chains[i].s = (i == 0 || !side) ? st : side->stream[i - 1];
    if (side && n_chains > 1) {
        HIP_TRY(hipEventRecord(side->fork, st));
        for (int i = 1; i < n_chains; ++i) HIP_TRY(hipStreamWaitEvent(chains[i].s, side->fork, 0));
    }
    const int T = chains[0].hd->T;
    for (int i = 0; i < n_chains; ++i) {
        Chain& ch = chains[i];
        float* slot_T = ch.path ? ch.path + (int64_t)T * ch.path_stride : nullptr;
        HIP_TRY(launch_init_x(ch.ws.x, ch.ws.acc, ch.n, ch.hd->D, T, seed, ch.row_offset, ch.row_stride, ch.row_shift,
                              ch.rng_stream, ch.init_norm, ch.path_write ? nullptr : slot_T,
                              ch.path_write ? slot_T : nullptr, ch.s));
        HIP_TRY(cond_embed(ch.hd, ch.z, ch.ws, ch.n * ch.hd->reps, ch.s));
    }
    for (int t = T; t >= 1; --t) {
        for (int i = 0; i < n_chains; ++i) {
            Chain& ch = chains[i];
            const int k = (T - t) % ch.ws.tb;
            const int64_t nh = ch.n * ch.hd->reps;      // rows of the head's activations
            if (k == 0) HIP_TRY(batch_stage(ch.hd, ch.ws, t, t < ch.ws.tb ? t : ch.ws.tb, nh, ch.s));
            HIP_TRY(head_body(ch.hd, ch.ws, k, nh, ch.s));
            TransArgs f = trans_args(ch.hd, ch.ws, t, ch.n);
            f.seed = seed; f.row_offset = ch.row_offset; f.tau = tau;
            f.row_stride = ch.row_stride; f.row_shift = ch.row_shift; f.rng_stream = ch.rng_stream;
            f.summary = ch.summary; f.is_target = ch.is_target; f.tokens = ch.tokens;
            f.path_mode = ch.path_mode; f.x0_own = ch.x0_own;
            if (ch.path && t >= 2) {
                float* slot = ch.path + (int64_t)(t - 1) * ch.path_stride;
                if (ch.path_write) f.path_out = slot; else f.path_in = slot;
            }
            HIP_TRY(launch_transition(f, ch.s));
        }
    }
    if (side && n_chains > 1) {
        for (int i = 1; i < n_chains; ++i) {
            HIP_TRY(hipEventRecord(side->join[i], chains[i].s));
            HIP_TRY(hipStreamWaitEvent(st, side->join[i], 0));
        }
    }
    return CSD_OK;
}

// argument checks shared by the denoising entry points
int check_ws(const char* who, const void* workspace, size_t have, size_t need) {
    if (!workspace) return fail(CSD_EINVAL, "%s: NULL buffer", who);
    if (((uintptr_t)workspace & 255u) != 0) return fail(CSD_EINVAL, "%s: workspace must be 256-byte aligned", who);
    if (have < need) return fail(CSD_EINVAL, "%s: workspace of %zu bytes, need %zu", who, have, need);
    return CSD_OK;
}

// One head alone over n contiguous local rows (chunked into chains).
int run_single_head(const csd_head* hd, const float* z, int64_t n, uint64_t seed, uint64_t row_offset,
                    int64_t row_stride, int64_t row_shift, int rng_stream, float tau, float* summary, int is_target,
                    float* tokens, void* workspace, hipStream_t st, Chain* chains, int* n_chains_out) {
    SideStreams* side = side_streams(hd->device);
    int64_t chunk_rows;
    const int n_chunks = plan_chunks(n, side != nullptr, &chunk_rows);
    char* wp = (char*)workspace;
    for (int c = 0; c < n_chunks; ++c) {
        const int64_t r0 = c * chunk_rows, m = (n - r0 < chunk_rows) ? n - r0 : chunk_rows;
        Chain& ch = chains[c];
        ch.hd = hd; ch.n = m; ch.z = z + r0 * hd->reps * hd->C;
        ch.row_offset = row_offset + (uint64_t)(r0 * row_stride); ch.row_stride = row_stride; ch.row_shift = row_shift;
        ch.rng_stream = rng_stream; ch.is_target = is_target;
        ch.summary = summary ? summary + r0 * row_stride * (5 * hd->D + 1) : nullptr;
        ch.tokens = tokens ? tokens + r0 * hd->D : nullptr;
        wp = carve(hd, m, steps_per_batch(hd, n), wp, &ch.ws);
    }
    *n_chains_out = n_chunks;
    return run_chains(chains, n_chunks, seed, tau, st, side);
}

// Both heads over the R rows of a call, cut into independent chains - (row chunk, head): rows
// never interact, and the two heads only share the noise, which each regenerates from the
// counters.  ratio_mode CSD_RATIO_ALIGNED is the method; the two others are the comparison
// modes of Table 1.  In the single-path mode the target follows the draft's stored path, so the
// draft's chains run to the end before the target's start.  x0_own (optional, [R,D]) takes the
// target's own final sample.
int run_pair(const csd_head* draft, const csd_head* target, const float* z_q, const float* z_p, int64_t R,
             uint64_t seed, uint64_t row_offset, float tau, int ratio_mode, float* summary, float* x0_own,
             float* path, char* wp, hipStream_t st) {
    const int D = draft->D, T = draft->T;
    SideStreams* side = side_streams(draft->device);
    int64_t chunk_rows;
    const int n_chunks = plan_chunks(R, side != nullptr, &chunk_rows);
    Chain chains[8] = {};
    int n_chains = 0;
    for (int c = 0; c < n_chunks; ++c) {
        const int64_t r0 = c * chunk_rows, n = (R - r0 < chunk_rows) ? R - r0 : chunk_rows;
        for (int which = 0; which < 2; ++which) {
            Chain& ch = chains[n_chains++];
            ch.hd = which ? target : draft; ch.n = n; ch.z = (which ? z_p : z_q) + r0 * ch.hd->reps * ch.hd->C;
            ch.row_offset = row_offset + (uint64_t)r0; ch.row_stride = 1; ch.row_shift = 0; ch.rng_stream = CSD_STREAM_TRAJ;
            ch.summary = summary + r0 * (5 * D + 1); ch.is_target = which; ch.tokens = nullptr;
            if (which && x0_own) ch.x0_own = x0_own + r0 * D;
            if (ratio_mode == CSD_RATIO_UNALIGNED) {
                ch.path_mode = PATH_OWN; ch.init_norm = 1;
                if (which) ch.rng_stream = CSD_STREAM_TRAJ_P;
            } else if (ratio_mode == CSD_RATIO_SINGLE_PATH) {
                ch.path_mode = which ? PATH_FOLLOW : PATH_OWN;
                ch.path = path + r0 * D; ch.path_stride = R * D; ch.path_write = !which;
            }
            wp = carve(ch.hd, n, steps_per_batch(ch.hd, R), wp, &ch.ws);
        }
    }
    if (ratio_mode == CSD_RATIO_SINGLE_PATH) {
        Chain half[4];
        for (int which = 0; which < 2; ++which) {
            for (int c = 0; c < n_chunks; ++c) half[c] = chains[2 * c + which];
            int rc = run_chains(half, n_chunks, seed, tau, st, side);
            if (rc != CSD_OK) return rc;
        }
    } else {
        int rc = run_chains(chains, n_chains, seed, tau, st, side);
        if (rc != CSD_OK) return rc;
    }
    (void)T;
    const float ref_diff = (float)(draft->ref_log_sigma - target->ref_log_sigma);
    for (int i = 0; i < n_chains; i += 2)
        HIP_TRY(launch_finish_summary(chains[i].summary, chains[i].ws.acc, chains[i + 1].ws.acc, ref_diff, chains[i].n, D,
                                      0, 1, 0, st));
    return CSD_OK;
}

int check_pair(const char* who, const csd_head* draft, const csd_head* target, int64_t n_groups, int gamma, float temperature) {
    if (!draft || !target) return fail(CSD_EINVAL, "%s: NULL head", who);
    if (n_groups < 0 || gamma < 1) return fail(CSD_EINVAL, "%s: n_groups >= 0 and gamma >= 1 required", who);
    if (draft->D != target->D || draft->T != target->T || draft->device != target->device || draft->C != target->C)
        return fail(CSD_EINVAL, "%s: heads must share token_dim, cond_dim, n_steps and device", who);
    if (!(temperature > 0.f)) return fail(CSD_EINVAL, "%s: temperature must be > 0", who);
    if (n_groups > (int64_t)(1 << 22) / gamma) return fail(CSD_EINVAL, "%s: more than 2^22 rows in one call", who);
    return CSD_OK;
}

}  // namespace

extern "C" {

const char* csd_last_error(void) { return g_err.c_str(); }

size_t csd_param_count(const csd_head_cfg_t* cfg) {
    const char* why;
    if (!cfg_ok(cfg, &why)) { g_err = why; return 0; }
    return param_count(cfg);
}

void csd_free_head(csd_head_t* h) {
    if (!h) return;
    DeviceGuard dg(h->device);
    (void)hipDeviceSynchronize();
    if (h->d_weights) (void)hipFree(h->d_weights);
    if (h->d_weights16) (void)hipFree(h->d_weights16);
    if (h->d_time_emb) (void)hipFree(h->d_time_emb);
    if (h->d_out_pad) (void)hipFree(h->d_out_pad);
    if (h->d_in_t) (void)hipFree(h->d_in_t);
    if (h->d_mod_all) (void)hipFree(h->d_mod_all);
    if (h->d_mod_all_bias) (void)hipFree(h->d_mod_all_bias);
    delete h;
}

int csd_set_guidance(csd_head_t* head, int32_t enabled, float scale) {
    if (!head) return fail(CSD_EINVAL, "csd_set_guidance: NULL head");
    if (enabled && !(scale == scale && scale >= -64.f && scale <= 64.f))
        return fail(CSD_EINVAL, "csd_set_guidance: scale must be a number in [-64, 64]");
    head->reps = enabled ? 2 : 1;
    head->cfg_scale = enabled ? scale : 0.f;
    return CSD_OK;
}

int csd_init_head(const csd_head_cfg_t* cfg, const float* weights_host, size_t n_floats, int device,
                  csd_head_t** out) {
    const char* why = "";
    if (!out) return fail(CSD_EINVAL, "csd_init_head: out is NULL");
    *out = nullptr;
    if (!cfg_ok(cfg, &why)) return fail(CSD_EINVAL, "csd_init_head: %s", why);
    if (!weights_host) return fail(CSD_EINVAL, "csd_init_head: weights_host is NULL");
    if (n_floats != param_count(cfg))
        return fail(CSD_EINVAL, "csd_init_head: n_floats = %zu, config needs %zu", n_floats, param_count(cfg));
    int n_dev = 0;
    HIP_TRY(hipGetDeviceCount(&n_dev));
    if (device < 0 || device >= n_dev) return fail(CSD_EINVAL, "csd_init_head: device %d of %d", device, n_dev);

    csd_head* h = new (std::nothrow) csd_head();
    if (!h) return fail(CSD_ENOMEM, "csd_init_head: host allocation failed");
    h->cfg = *cfg; h->cfg.alpha_bar = nullptr; h->device = device;
    h->D = cfg->token_dim; h->C = cfg->cond_dim; h->W = cfg->width; h->L = cfg->n_blocks; h->T = cfg->n_steps;
    h->ln_eps = cfg->ln_eps > 0.f ? cfg->ln_eps : 1e-6f;
    const int D = h->D, C = h->C, W = h->W, L = h->L, T = h->T;

    // ---- schedule constants in double (Eq. 3 with the learned-range variance)
    std::vector<double> abar(T + 1, 1.0);
    if (cfg->schedule == CSD_TABLE) {
        for (int t = 0; t <= T; ++t) abar[t] = cfg->alpha_bar[t];
        bool ok = abar[0] == 1.0;
        for (int t = 1; t <= T && ok; ++t) ok = abar[t] > 0.0 && abar[t] < abar[t - 1];
        if (!ok) { delete h; return fail(CSD_EINVAL, "csd_init_head: alpha_bar must start at 1 and decrease strictly within (0,1]"); }
    } else {
        auto f = [&](int t) { const double c = std::cos((((double)t / T) + 0.008) / 1.008 * M_PI / 2.0); return c * c; };
        for (int t = 1; t <= T; ++t) {
            const double b = std::fmin(1.0 - f(t) / f(t - 1), 0.999);
            abar[t] = abar[t - 1] * (1.0 - b);
        }
    }
    h->coef.assign(T + 1, StepCoef{0, 0, 0, 0});
    std::vector<double> lbt(T + 2, 0.0), lb(T + 2, 0.0);
    for (int t = 1; t <= T; ++t) {
        const double alpha = abar[t] / abar[t - 1], beta = 1.0 - alpha;
        lb[t] = std::log(beta);
        if (t >= 2) lbt[t] = std::log(beta * (1.0 - abar[t - 1]) / (1.0 - abar[t]));
    }
    lbt[1] = (T >= 2) ? lbt[2] : lb[1];       // posterior variance is 0 at t = 1: clipped to the next one
    h->ref_log_sigma = 0.0;
    for (int t = 1; t <= T; ++t) {
        // every sampler here is mu = a x_t + b eps_hat, log sigma^2 = lmid + v lhalf; with the skip
        // eps_hat = gain sqrt(1-abar_t) x_t + o the kernels use mu = cx x_t - co o
        const double alpha = abar[t] / abar[t - 1], beta = 1.0 - alpha;
        double a = 1.0 / std::sqrt(alpha), b, lmid, lhalf;
        if (cfg->sampler == CSD_SAMPLER_DDIM) {
            const double var = (double)cfg->ddim_eta * (double)cfg->ddim_eta * std::exp(lbt[t]);
            b = std::sqrt(std::fmax(0.0, 1.0 - abar[t - 1] - var)) - std::sqrt(1.0 - abar[t]) / std::sqrt(alpha);
            lmid = std::log(var); lhalf = 0.0;
        } else {
            b = -beta / (std::sqrt(1.0 - abar[t]) * std::sqrt(alpha));
            lmid = 0.5 * (lb[t] + lbt[t]); lhalf = 0.5 * (lb[t] - lbt[t]);
        }
        const double cx = a + b * (double)cfg->eps_skip_gain * std::sqrt(1.0 - abar[t]);
        h->coef[t] = StepCoef{(float)cx, (float)(-b), (float)lmid, (float)lhalf};
        if (t >= 2) h->ref_log_sigma += 0.5 * D * lmid;
    }
    h->skip_sqrt.assign(T + 1, 0.f);
    for (int t = 1; t <= T; ++t) h->skip_sqrt[t] = (float)((double)cfg->eps_skip_gain * std::sqrt(1.0 - abar[t]));

    DeviceGuard dg(device);
    if (!dg.ok) { delete h; return fail(CSD_EHIP, "csd_init_head: cannot select device %d", device); }
    int rc = CSD_OK;
    float* d_feats = nullptr; float* d_tmp = nullptr;
    auto bail = [&](int code) { if (d_feats) (void)hipFree(d_feats); if (d_tmp) (void)hipFree(d_tmp); csd_free_head(h); return code; };
#define INIT_TRY(expr)                                                                                  \
    do { hipError_t e_ = (expr);                                                                        \
         if (e_ != hipSuccess) {                                                                        \
             rc = fail(e_ == hipErrorOutOfMemory ? CSD_ENOMEM : CSD_EHIP, "csd_init_head: %s: %s", #expr, \
                       hipGetErrorString(e_));                                                          \
             return bail(rc); } } while (0)

    INIT_TRY(hipMalloc((void**)&h->d_weights, n_floats * sizeof(float)));
    INIT_TRY(hipMemcpy(h->d_weights, weights_host, n_floats * sizeof(float), hipMemcpyHostToDevice));

    // ---- carve the blob into layers (order documented in csd.h)
    size_t off = 0, n16 = 0;
    const bool b16 = cfg->gemm_dtype == CSD_BF16;
    std::vector<Linear*> big;     // layers that get a bf16 copy
    auto lin = [&](Linear& l, int n_out, int n_in, bool is_big) {
        l.n_out = n_out; l.n_in = n_in;
        l.w = h->d_weights + off; off += (size_t)n_out * n_in;
        l.b = h->d_weights + off; off += (size_t)n_out;
        if (is_big && b16) { big.push_back(&l); n16 += (size_t)n_out * n_in; }
    };
    h->mod.resize(L); h->fc1.resize(L); h->fc2.resize(L);
    lin(h->t1, W, CSD_TIME_FEATURES, false);
    lin(h->t2, W, W, false);
    lin(h->cond, W, C, false);
    lin(h->in, W, D, false);
    for (int l = 0; l < L; ++l) { lin(h->mod[l], 3 * W, W, true); lin(h->fc1[l], W, W, true); lin(h->fc2[l], W, W, true); }
    lin(h->fmod, 2 * W, W, true);
    lin(h->out, 2 * D, W, false);
    if (off != n_floats) return bail(fail(CSD_EINVAL, "csd_init_head: internal layout mismatch"));
    // input projection transposed to [D, W] (host transpose of the caller's blob)
    {
        const float* w_in_host = weights_host + ((size_t)W * CSD_TIME_FEATURES + W + (size_t)W * W + W + (size_t)W * C + W);
        std::vector<float> tr((size_t)D * W);
        for (int o = 0; o < W; ++o)
            for (int d = 0; d < D; ++d) tr[(size_t)d * W + o] = w_in_host[(size_t)o * D + d];
        INIT_TRY(hipMalloc((void**)&h->d_in_t, tr.size() * sizeof(float)));
        INIT_TRY(hipMemcpy(h->d_in_t, tr.data(), tr.size() * sizeof(float), hipMemcpyHostToDevice));
    }
    // output layer padded with zero rows to 64 outputs, so that it runs through the GEMM kernels
    {
        const size_t nw = (size_t)64 * W;
        INIT_TRY(hipMalloc((void**)&h->d_out_pad, (nw + 64) * sizeof(float)));
        INIT_TRY(hipMemset(h->d_out_pad, 0, (nw + 64) * sizeof(float)));
        INIT_TRY(hipMemcpy(h->d_out_pad, h->out.w, (size_t)2 * D * W * sizeof(float), hipMemcpyDeviceToDevice));
        INIT_TRY(hipMemcpy(h->d_out_pad + nw, h->out.b, (size_t)2 * D * sizeof(float), hipMemcpyDeviceToDevice));
        h->out_pad.w = h->d_out_pad; h->out_pad.b = h->d_out_pad + nw; h->out_pad.n_out = 64; h->out_pad.n_in = W;
        if (b16) n16 += 2 * nw;
    }
    if (b16) {
        INIT_TRY(hipMalloc((void**)&h->d_weights16, n16 * sizeof(bf16_t)));
        size_t o16 = 0;
        for (Linear* l : big) {
            const size_t n = (size_t)l->n_out * l->n_in;
            INIT_TRY(launch_f32_to_bf16(l->w, h->d_weights16 + o16, n, nullptr));
            l->w16 = h->d_weights16 + o16; o16 += n;
        }
        // [w | w]: row o of the bf16 output layer holds its W weights twice
        bf16_t* dst = h->d_weights16 + o16;
        INIT_TRY(launch_f32_to_bf16_rows(h->out_pad.w, dst, 64, W, 2 * W, nullptr));
        INIT_TRY(launch_f32_to_bf16_rows(h->out_pad.w, dst + W, 64, W, 2 * W, nullptr));
        h->out_pad.w16 = dst;
        // K = 2W of the output projection in 4 ranges where each is a whole number of 64-wide slabs
        const char* e = getenv("CSD_OUT_SPLITS");
        const int want = (e && *e) ? atoi(e) : 4;
        h->out_splits = (want >= 1 && want <= 8 && (2 * W) % (64 * want) == 0 && 2 * W >= 1024) ? want : 1;
    }

    // ---- the L modulation layers stacked into one [L*3W, W] matrix: they all read the same
    // s = SiLU(E_t + e) and do not depend on the trajectory, so one GEMM per step serves them all
    {
        const size_t per = (size_t)3 * W * W, nb = (size_t)3 * W;
        INIT_TRY(hipMalloc(&h->d_mod_all, (size_t)L * per * (b16 ? sizeof(bf16_t) : sizeof(float))));
        INIT_TRY(hipMalloc((void**)&h->d_mod_all_bias, (size_t)L * nb * sizeof(float)));
        for (int l = 0; l < L; ++l) {
            if (b16) INIT_TRY(hipMemcpy((bf16_t*)h->d_mod_all + l * per, h->mod[l].w16, per * sizeof(bf16_t), hipMemcpyDeviceToDevice));
            else INIT_TRY(hipMemcpy((float*)h->d_mod_all + l * per, h->mod[l].w, per * sizeof(float), hipMemcpyDeviceToDevice));
            INIT_TRY(hipMemcpy(h->d_mod_all_bias + l * nb, h->mod[l].b, nb * sizeof(float), hipMemcpyDeviceToDevice));
        }
        h->mod_all.w = b16 ? nullptr : (const float*)h->d_mod_all;
        h->mod_all.w16 = b16 ? (const bf16_t*)h->d_mod_all : nullptr;
        h->mod_all.b = h->d_mod_all_bias; h->mod_all.n_out = L * 3 * W; h->mod_all.n_in = W;
    }

    // ---- time embedding table E_t[t], t = 1..T: sinusoidal features in double on the
    // host (a constant table), the two linear layers on the device in fp32
    {
        const int F = CSD_TIME_FEATURES, half = F / 2;
        const double t_scale = cfg->t_scale > 0.f ? (double)cfg->t_scale : 1000.0 / T;
        std::vector<float> feats((size_t)T * F);
        for (int t = 1; t <= T; ++t)
            for (int i = 0; i < half; ++i) {
                const double a = t_scale * (t - 1) * std::exp(-std::log(10000.0) * i / half);
                feats[(size_t)(t - 1) * F + i] = (float)std::cos(a);
                feats[(size_t)(t - 1) * F + half + i] = (float)std::sin(a);
            }
        INIT_TRY(hipMalloc((void**)&d_feats, feats.size() * sizeof(float)));
        INIT_TRY(hipMalloc((void**)&d_tmp, (size_t)T * W * sizeof(float)));
        INIT_TRY(hipMalloc((void**)&h->d_time_emb, (size_t)(T + 1) * W * sizeof(float)));
        INIT_TRY(hipMemcpy(d_feats, feats.data(), feats.size() * sizeof(float), hipMemcpyHostToDevice));
        INIT_TRY(hipMemset(h->d_time_emb, 0, (size_t)W * sizeof(float)));
        GemmArgs g{};
        g.A = d_feats; g.lda = F; g.B = h->t1.w; g.bias = h->t1.b; g.C = d_tmp; g.ldc = W;
        g.M = T; g.N = W; g.K = F; g.epi = EPI_BIAS_SILU;
        INIT_TRY(launch_gemm_f32(g, nullptr));
        g.A = d_tmp; g.lda = W; g.B = h->t2.w; g.bias = h->t2.b; g.C = h->d_time_emb + W; g.K = W; g.epi = EPI_BIAS;
        INIT_TRY(launch_gemm_f32(g, nullptr));
    }
    INIT_TRY(hipDeviceSynchronize());
    (void)hipFree(d_feats); (void)hipFree(d_tmp);
#undef INIT_TRY
    *out = h;
    return CSD_OK;
}

size_t csd_workspace_bytes(const csd_head_t* draft, const csd_head_t* target, int64_t n_rows) {
    if (n_rows < 0 || (!draft && !target)) return 0;
    // the row chunks of a call (see plan_chunks) add up to n_rows; every buffer of every chunk is
    // aligned to 256 bytes, which the slack covers (up to 4 chunks x 11 buffers)
    size_t n = 256;
    if (draft) n += head_ws_bytes(draft, n_rows, steps_per_batch(draft, n_rows)) + 4 * 16 * 256;
    if (target) n += head_ws_bytes(target, n_rows, steps_per_batch(target, n_rows)) + 4 * 16 * 256;
    return n;
}

int csd_denoise_lockstep(const csd_head_t* draft, const csd_head_t* target, const float* z_q, const float* z_p,
                         int64_t n_groups, int32_t gamma, uint64_t seed, uint64_t row_offset, float temperature,
                         float* summary, void* workspace, size_t workspace_bytes, void* hip_stream) {
    int rc = check_pair("csd_denoise_lockstep", draft, target, n_groups, gamma, temperature);
    if (rc != CSD_OK) return rc;
    const int64_t R = n_groups * gamma;
    if (R == 0) return CSD_OK;
    if (!z_q || !z_p || !summary) return fail(CSD_EINVAL, "csd_denoise_lockstep: NULL buffer");
    rc = check_ws("csd_denoise_lockstep", workspace, workspace_bytes, csd_workspace_bytes(draft, target, R));
    if (rc != CSD_OK) return rc;
    return run_pair(draft, target, z_q, z_p, R, seed, row_offset, temperature, CSD_RATIO_ALIGNED, summary, nullptr,
                    nullptr, (char*)workspace, (hipStream_t)hip_stream);
}

size_t csd_ablation_workspace_bytes(const csd_head_t* draft, const csd_head_t* target, int64_t n_rows, int32_t ratio_mode) {
    if (n_rows < 0 || !draft || !target) return 0;
    size_t n = csd_workspace_bytes(draft, target, n_rows) + align_up((size_t)n_rows * draft->D * 4, 256);
    if (ratio_mode == CSD_RATIO_SINGLE_PATH) n += align_up((size_t)(draft->T + 1) * n_rows * draft->D * 4, 256);
    return n;
}

int csd_denoise_ablation(const csd_head_t* draft, const csd_head_t* target, const float* z_q, const float* z_p,
                         int64_t n_groups, int32_t gamma, uint64_t seed, uint64_t row_offset, float temperature,
                         int32_t ratio_mode, float* summary, float* dist2, void* workspace, size_t workspace_bytes,
                         void* hip_stream) {
    int rc = check_pair("csd_denoise_ablation", draft, target, n_groups, gamma, temperature);
    if (rc != CSD_OK) return rc;
    if (ratio_mode != CSD_RATIO_ALIGNED && ratio_mode != CSD_RATIO_UNALIGNED && ratio_mode != CSD_RATIO_SINGLE_PATH)
        return fail(CSD_EINVAL, "csd_denoise_ablation: unknown ratio_mode %d", (int)ratio_mode);
    const int64_t R = n_groups * gamma;
    if (R == 0) return CSD_OK;
    if (!z_q || !z_p || !summary || !dist2) return fail(CSD_EINVAL, "csd_denoise_ablation: NULL buffer");
    rc = check_ws("csd_denoise_ablation", workspace, workspace_bytes, csd_ablation_workspace_bytes(draft, target, R, ratio_mode));
    if (rc != CSD_OK) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    char* wp = (char*)workspace;
    float* x0_own = (float*)wp; wp += align_up((size_t)R * draft->D * 4, 256);
    float* path = nullptr;
    if (ratio_mode == CSD_RATIO_SINGLE_PATH) { path = (float*)wp; wp += align_up((size_t)(draft->T + 1) * R * draft->D * 4, 256); }
    rc = run_pair(draft, target, z_q, z_p, R, seed, row_offset, temperature, ratio_mode, summary, x0_own, path, wp, st);
    if (rc != CSD_OK) return rc;
    HIP_TRY(launch_token_distance(summary, x0_own, dist2, R, draft->D, st));
    return CSD_OK;
}

int csd_denoise_draft(const csd_head_t* draft, const float* z_q, int64_t n_groups, int32_t gamma, int32_t position,
                      uint64_t seed, uint64_t row_offset, float temperature, float* summary, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
    if (!draft) return fail(CSD_EINVAL, "csd_denoise_draft: NULL head");
    if (n_groups < 0 || gamma < 1 || position < 0 || position >= gamma)
        return fail(CSD_EINVAL, "csd_denoise_draft: n_groups >= 0, gamma >= 1 and 0 <= position < gamma required");
    if (!(temperature > 0.f)) return fail(CSD_EINVAL, "csd_denoise_draft: temperature must be > 0");
    if (n_groups > (int64_t)(1 << 22) / gamma) return fail(CSD_EINVAL, "csd_denoise_draft: more than 2^22 rows in one call");
    if (n_groups == 0) return CSD_OK;
    if (!z_q || !summary) return fail(CSD_EINVAL, "csd_denoise_draft: NULL buffer");
    int rc = check_ws("csd_denoise_draft", workspace, workspace_bytes, csd_workspace_bytes(draft, nullptr, n_groups));
    if (rc != CSD_OK) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    Chain chains[8] = {};
    int n_chains = 0;
    rc = run_single_head(draft, z_q, n_groups, seed, row_offset, gamma, position, CSD_STREAM_TRAJ, temperature, summary, 0,
                         nullptr, workspace, st, chains, &n_chains);
    if (rc != CSD_OK) return rc;
    for (int i = 0; i < n_chains; ++i)      // park the draft's half of log Sigma in the last column
        HIP_TRY(launch_finish_summary(chains[i].summary, chains[i].ws.acc, nullptr, 0.f, chains[i].n, draft->D, 1,
                                      gamma, position, st));
    return CSD_OK;
}

int csd_denoise_target(const csd_head_t* target, const csd_head_t* draft, const float* z_p, int64_t n_groups,
                       int32_t gamma, uint64_t seed, uint64_t row_offset, float temperature, float* summary,
                       void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!target || !draft) return fail(CSD_EINVAL, "csd_denoise_target: NULL head");
    if (n_groups < 0 || gamma < 1) return fail(CSD_EINVAL, "csd_denoise_target: n_groups >= 0 and gamma >= 1 required");
    if (draft->D != target->D || draft->T != target->T || draft->device != target->device)
        return fail(CSD_EINVAL, "csd_denoise_target: heads must share token_dim, n_steps and device");
    if (!(temperature > 0.f)) return fail(CSD_EINVAL, "csd_denoise_target: temperature must be > 0");
    if (n_groups > (int64_t)(1 << 22) / gamma) return fail(CSD_EINVAL, "csd_denoise_target: more than 2^22 rows in one call");
    const int64_t R = n_groups * gamma;
    if (R == 0) return CSD_OK;
    if (!z_p || !summary) return fail(CSD_EINVAL, "csd_denoise_target: NULL buffer");
    int rc = check_ws("csd_denoise_target", workspace, workspace_bytes, csd_workspace_bytes(nullptr, target, R));
    if (rc != CSD_OK) return rc;
    hipStream_t st = (hipStream_t)hip_stream;
    Chain chains[8] = {};
    int n_chains = 0;
    rc = run_single_head(target, z_p, R, seed, row_offset, 1, 0, CSD_STREAM_TRAJ, temperature, summary, 1, nullptr,
                         workspace, st, chains, &n_chains);
    if (rc != CSD_OK) return rc;
    const float ref_diff = (float)(draft->ref_log_sigma - target->ref_log_sigma);
    for (int i = 0; i < n_chains; ++i)
        HIP_TRY(launch_finish_summary(chains[i].summary, nullptr, chains[i].ws.acc, ref_diff, chains[i].n, target->D, 2,
                                      1, 0, st));
    return CSD_OK;
}

int csd_sample(const csd_head_t* head, const float* z, int64_t n_rows, uint64_t seed, uint64_t row_offset,
               int32_t rng_stream, float temperature, float* tokens, void* workspace, size_t workspace_bytes,
               void* hip_stream) {
    if (!head) return fail(CSD_EINVAL, "csd_sample: NULL head");
    if (n_rows < 0 || n_rows > (1 << 22)) return fail(CSD_EINVAL, "csd_sample: n_rows out of range");
    if (rng_stream != CSD_STREAM_TRAJ && rng_stream != CSD_STREAM_BONUS)
        return fail(CSD_EINVAL, "csd_sample: rng_stream must be CSD_STREAM_TRAJ or CSD_STREAM_BONUS");
    if (!(temperature > 0.f)) return fail(CSD_EINVAL, "csd_sample: temperature must be > 0");
    if (n_rows == 0) return CSD_OK;
    if (!z || !tokens) return fail(CSD_EINVAL, "csd_sample: NULL buffer");
    int rc = check_ws("csd_sample", workspace, workspace_bytes, csd_workspace_bytes(head, nullptr, n_rows));
    if (rc != CSD_OK) return rc;
    Chain chains[8] = {};
    int n_chains = 0;
    return run_single_head(head, z, n_rows, seed, row_offset, 1, 0, rng_stream, temperature, nullptr, 0, tokens, workspace,
                           (hipStream_t)hip_stream, chains, &n_chains);
}

int csd_append_bonus(float* tokens, int32_t* n_out, const int32_t* n_accept, const float* bonus, int64_t n_groups,
                     int32_t gamma, int32_t token_dim, void* hip_stream) {
    if (n_groups < 0 || gamma < 1 || gamma > 64) return fail(CSD_EINVAL, "csd_append_bonus: n_groups >= 0 and 1 <= gamma <= 64 required");
    if (token_dim != 4 && token_dim != 8 && token_dim != 16) return fail(CSD_EINVAL, "csd_append_bonus: token_dim must be 4, 8 or 16");
    if (n_groups == 0) return CSD_OK;
    if (!tokens || !n_out || !n_accept || !bonus) return fail(CSD_EINVAL, "csd_append_bonus: NULL buffer");
    HIP_TRY(launch_append_bonus(tokens, n_out, n_accept, bonus, n_groups, gamma, token_dim, (hipStream_t)hip_stream));
    return CSD_OK;
}

namespace {
int check_gmm(const char* who, int64_t n, int gamma, int K, int D) {
    if (n < 0 || gamma < 1 || gamma > 64) return fail(CSD_EINVAL, "%s: n >= 0 and 1 <= gamma <= 64 required", who);
    if (K < 1 || K > 64) return fail(CSD_EINVAL, "%s: 1 <= n_components <= 64 required", who);
    if (!(D == 4 || D == 8 || D == 16)) return fail(CSD_EINVAL, "%s: token_dim must be 4, 8 or 16", who);
    if (n > (int64_t)1 << 30) return fail(CSD_EINVAL, "%s: too many rows", who);
    return CSD_OK;
}
}  // namespace

int csd_gmm_draft_sample(const float* pi_q, const float* mu_q, const float* logvar_q, int64_t n_rows,
                         int32_t n_components, int32_t token_dim, uint64_t seed, uint64_t row_offset, float* x,
                         void* hip_stream) {
    int rc = check_gmm("csd_gmm_draft_sample", n_rows, 1, n_components, token_dim);
    if (rc != CSD_OK) return rc;
    if (n_rows == 0) return CSD_OK;
    if (!pi_q || !mu_q || !logvar_q || !x) return fail(CSD_EINVAL, "csd_gmm_draft_sample: NULL buffer");
    HIP_TRY(launch_gmm_draft_sample(pi_q, mu_q, logvar_q, n_rows, n_components, token_dim, seed, row_offset, x,
                                    (hipStream_t)hip_stream));
    return CSD_OK;
}

int csd_gmm_verify(const float* x, const float* pi_p, const float* mu_p, const float* logvar_p, const float* pi_q,
                   const float* mu_q, const float* logvar_q, int64_t n_groups, int32_t gamma, int32_t n_components,
                   int32_t token_dim, uint64_t seed, uint64_t row_offset, int32_t* n_accept, float* log_ratio,
                   uint8_t* accept_mask, void* hip_stream) {
    int rc = check_gmm("csd_gmm_verify", n_groups, gamma, n_components, token_dim);
    if (rc != CSD_OK) return rc;
    if (n_groups == 0) return CSD_OK;
    if (!x || !pi_p || !mu_p || !logvar_p || !pi_q || !mu_q || !logvar_q || !n_accept)
        return fail(CSD_EINVAL, "csd_gmm_verify: NULL buffer");
    HIP_TRY(launch_gmm_verify(x, pi_p, mu_p, logvar_p, pi_q, mu_q, logvar_q, n_groups, gamma, n_components, token_dim,
                              seed, row_offset, n_accept, log_ratio, accept_mask, (hipStream_t)hip_stream));
    return CSD_OK;
}

int csd_gmm_resample(const float* x, const int32_t* n_accept, const float* pi_p, const float* mu_p,
                     const float* logvar_p, const float* pi_q, const float* mu_q, const float* logvar_q,
                     int64_t n_groups, int32_t gamma, int32_t n_components, int32_t token_dim, uint64_t seed,
                     uint64_t row_offset, int32_t max_trips, float* tokens, int32_t* n_out, int32_t* trips,
                     uint32_t* flags, void* hip_stream) {
    int rc = check_gmm("csd_gmm_resample", n_groups, gamma, n_components, token_dim);
    if (rc != CSD_OK) return rc;
    if (max_trips < 1 || max_trips > 65534) return fail(CSD_EINVAL, "csd_gmm_resample: 1 <= max_trips <= 65534 required");
    if (n_groups == 0) return CSD_OK;
    if (!x || !n_accept || !pi_p || !mu_p || !logvar_p || !pi_q || !mu_q || !logvar_q || !tokens || !n_out)
        return fail(CSD_EINVAL, "csd_gmm_resample: NULL buffer");
    HIP_TRY(launch_gmm_resample(x, n_accept, pi_p, mu_p, logvar_p, pi_q, mu_q, logvar_q, n_groups, gamma, n_components,
                                token_dim, seed, row_offset, max_trips, tokens, n_out, trips, flags,
                                (hipStream_t)hip_stream));
    return CSD_OK;
}

int csd_head_eval(const csd_head_t* head, const float* x, const float* z, int32_t t, int64_t n_rows, float* out,
                  void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!head) return fail(CSD_EINVAL, "csd_head_eval: NULL head");
    if (t < 1 || t > head->T) return fail(CSD_EINVAL, "csd_head_eval: t = %d outside 1..%d", t, head->T);
    if (n_rows < 0 || n_rows > (1 << 22)) return fail(CSD_EINVAL, "csd_head_eval: n_rows out of range");
    if (n_rows == 0) return CSD_OK;
    if (!x || !z || !out || !workspace) return fail(CSD_EINVAL, "csd_head_eval: NULL buffer");
    if (((uintptr_t)workspace & 255u) != 0) return fail(CSD_EINVAL, "csd_head_eval: workspace must be 256-byte aligned");
    if (workspace_bytes < csd_workspace_bytes(head, nullptr, n_rows))
        return fail(CSD_EINVAL, "csd_head_eval: workspace of %zu bytes, need %zu", workspace_bytes,
                    csd_workspace_bytes(head, nullptr, n_rows));
    hipStream_t st = (hipStream_t)hip_stream;
    HeadWs ws;
    carve(head, n_rows, steps_per_batch(head, n_rows), (char*)workspace, &ws);
    HIP_TRY(hipMemcpyAsync(ws.x, x, (size_t)n_rows * head->D * sizeof(float), hipMemcpyDeviceToDevice, st));
    HIP_TRY(cond_embed(head, z, ws, n_rows * head->reps, st));
    HIP_TRY(batch_stage(head, ws, t, 1, n_rows * head->reps, st));
    HIP_TRY(head_body(head, ws, 0, n_rows * head->reps, st));
    TransArgs f = trans_args(head, ws, t, n_rows);
    f.raw_out = out; f.skip_coef = head->skip_sqrt[t];
    HIP_TRY(launch_transition(f, st));
    return CSD_OK;
}

int csd_verify(const float* summary, int64_t n_groups, int32_t gamma, int32_t token_dim, uint64_t seed,
               uint64_t row_offset, float temperature, int32_t* n_accept, float* log_ratio, uint8_t* mask,
               void* hip_stream) {
    if (n_groups < 0 || gamma < 1 || gamma > 64) return fail(CSD_EINVAL, "csd_verify: n_groups >= 0 and 1 <= gamma <= 64 required");
    if (!(token_dim == 4 || token_dim == 8 || token_dim == 16)) return fail(CSD_EINVAL, "csd_verify: token_dim must be 4, 8 or 16");
    if (!(temperature > 0.f)) return fail(CSD_EINVAL, "csd_verify: temperature must be > 0");
    if (n_groups > (int64_t)1 << 30) return fail(CSD_EINVAL, "csd_verify: too many groups");
    if (n_groups == 0) return CSD_OK;
    if (!summary || !n_accept) return fail(CSD_EINVAL, "csd_verify: NULL buffer");
    HIP_TRY(launch_verify(summary, n_groups, gamma, token_dim, seed, row_offset, temperature, n_accept, log_ratio,
                          mask, (hipStream_t)hip_stream));
    return CSD_OK;
}

int csd_resample(const float* summary, const int32_t* n_accept, int64_t n_groups, int32_t gamma, int32_t token_dim,
                 uint64_t seed, uint64_t row_offset, float temperature, int32_t max_trips, float* tokens,
                 int32_t* n_out, int32_t* trips, uint32_t* flags, void* hip_stream) {
    if (n_groups < 0 || gamma < 1 || gamma > 64) return fail(CSD_EINVAL, "csd_resample: n_groups >= 0 and 1 <= gamma <= 64 required");
    if (!(token_dim == 4 || token_dim == 8 || token_dim == 16)) return fail(CSD_EINVAL, "csd_resample: token_dim must be 4, 8 or 16");
    if (!(temperature > 0.f)) return fail(CSD_EINVAL, "csd_resample: temperature must be > 0");
    if (max_trips < 1 || max_trips > 65535) return fail(CSD_EINVAL, "csd_resample: max_trips must be in [1,65535]");
    if (n_groups > (int64_t)1 << 30) return fail(CSD_EINVAL, "csd_resample: too many groups");
    if (n_groups == 0) return CSD_OK;
    if (!summary || !n_accept || !tokens || !n_out) return fail(CSD_EINVAL, "csd_resample: NULL buffer");
    HIP_TRY(launch_resample(summary, n_accept, n_groups, gamma, token_dim, seed, row_offset, temperature, max_trips,
                            tokens, n_out, trips, flags, (hipStream_t)hip_stream));
    return CSD_OK;
}

int csd_profile_enable(int32_t max_launches) {
    for (hipEvent_t ev : g_prof.ev) (void)hipEventDestroy(ev);
    g_prof.ev.clear(); g_prof.flops.clear(); g_prof.used = 0; g_prof.on = false;
    if (g_prof.d_pair) { (void)hipFree(g_prof.d_pair); g_prof.d_pair = nullptr; }
    if (max_launches <= 0) return CSD_OK;
    if (max_launches > (1 << 20)) return fail(CSD_EINVAL, "csd_profile_enable: at most 2^20 launches");
    g_prof.ev.resize((size_t)max_launches * 2);
    for (size_t i = 0; i < g_prof.ev.size(); ++i) {
        hipError_t e = hipEventCreate(&g_prof.ev[i]);
        if (e != hipSuccess) {
            for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(g_prof.ev[j]);
            g_prof.ev.clear();
            return fail(CSD_EHIP, "csd_profile_enable: hipEventCreate: %s", hipGetErrorString(e));
        }
    }
    // [start, end] per launch: start preset to all ones (atomicMin), end to zero (atomicMax)
    std::vector<unsigned long long> init((size_t)max_launches * 2);
    for (size_t i = 0; i < init.size(); i += 2) { init[i] = ~0ull; init[i + 1] = 0ull; }
    HIP_TRY(hipMalloc((void**)&g_prof.d_pair, init.size() * sizeof(unsigned long long)));
    HIP_TRY(hipMemcpy(g_prof.d_pair, init.data(), init.size() * sizeof(unsigned long long), hipMemcpyHostToDevice));
    g_prof.on = true;
    return CSD_OK;
}

int csd_profile_read(double* ms_sum, int64_t* launches, double* flops_sum, double* ms_sum_on_device) {
    if (!ms_sum || !launches || !flops_sum) return fail(CSD_EINVAL, "csd_profile_read: NULL output");
    double ms = 0.0, fl = 0.0;
    for (size_t i = 0; i < g_prof.used; ++i) {
        HIP_TRY(hipEventSynchronize(g_prof.ev[2 * i + 1]));
        float t = 0.f;
        HIP_TRY(hipEventElapsedTime(&t, g_prof.ev[2 * i], g_prof.ev[2 * i + 1]));
        ms += t; fl += g_prof.flops[i];
    }
    if (ms_sum_on_device) {
        *ms_sum_on_device = 0.0;
        if (g_prof.d_pair && g_prof.used) {
            std::vector<unsigned long long> ts(g_prof.used * 2);
            HIP_TRY(hipMemcpy(ts.data(), g_prof.d_pair, ts.size() * sizeof(unsigned long long), hipMemcpyDeviceToHost));
            double ticks = 0.0;
            bool all = true;
            for (size_t i = 0; i < g_prof.used; ++i) {
                if (ts[2 * i + 1] > ts[2 * i]) ticks += (double)(ts[2 * i + 1] - ts[2 * i]); else all = false;
            }
            *ms_sum_on_device = all ? ticks / 1e5 : 0.0;      // 100 MHz constant clock; 0 = not available (fp32 kernels)
            for (size_t i = 0; i < ts.size(); i += 2) { ts[i] = ~0ull; ts[i + 1] = 0ull; }
            HIP_TRY(hipMemcpy(g_prof.d_pair, ts.data(), ts.size() * sizeof(unsigned long long), hipMemcpyHostToDevice));
        }
    }
    *ms_sum = ms; *launches = (int64_t)g_prof.used; *flops_sum = fl;
    g_prof.used = 0; g_prof.flops.clear();
    return CSD_OK;
}

int csd_gemm_bf16(const void* A, const void* B, const float* bias, int64_t M, int32_t N, int32_t K, int32_t epilogue,
                  int32_t out_f32, void* C, const void* gate, void* hip_stream) {
    if (M < 0 || M > (1 << 22) || N < 64 || K < 64 || N % 64 || K % 64 || N > (1 << 20) || K > (1 << 20))
        return fail(CSD_EINVAL, "csd_gemm_bf16: shape out of range (N and K multiples of 64)");
    if (epilogue < 0 || epilogue > 2) return fail(CSD_EINVAL, "csd_gemm_bf16: epilogue must be 0, 1 or 2");
    if (M == 0) return CSD_OK;
    if (!A || !B || !bias || !C || (epilogue == EPI_GATE_RES && !gate)) return fail(CSD_EINVAL, "csd_gemm_bf16: NULL buffer");
    GemmArgs g{};
    g.A = A; g.lda = K; g.B = B; g.bias = bias; g.C = C; g.ldc = N; g.gate = gate; g.ldg = N;
    g.M = (int)M; g.N = N; g.K = K; g.epi = epilogue; g.c_is_f32 = out_f32 ? 1 : 0;
    HIP_TRY(launch_gemm_bf16(g, (hipStream_t)hip_stream));
    return CSD_OK;
}

int csd_rng_normals(uint64_t seed, uint64_t row_offset, int64_t n_rows, int32_t slot, int32_t stream_id,
                    int32_t n_cols, float* out, void* hip_stream) {
    if (n_rows < 0 || n_rows > ((int64_t)1 << 30) || slot < 0 || slot > 65535 || stream_id < 0 || stream_id > 65535 ||
        n_cols < 4 || n_cols % 4 || n_cols > 1024)
        return fail(CSD_EINVAL, "csd_rng_normals: argument out of range");
    if (n_rows == 0) return CSD_OK;
    if (!out) return fail(CSD_EINVAL, "csd_rng_normals: out is NULL");
    HIP_TRY(launch_rng_normals(seed, row_offset, n_rows, slot, stream_id, n_cols, out, (hipStream_t)hip_stream));
    return CSD_OK;
}

int csd_rng_uniforms(uint64_t seed, uint64_t row_offset, int64_t n_rows, int32_t slot, int32_t stream_id, float* out,
                     void* hip_stream) {
    if (n_rows < 0 || n_rows > ((int64_t)1 << 30) || slot < 0 || slot > 65535 || stream_id < 0 || stream_id > 65535)
        return fail(CSD_EINVAL, "csd_rng_uniforms: argument out of range");
    if (n_rows == 0) return CSD_OK;
    if (!out) return fail(CSD_EINVAL, "csd_rng_uniforms: out is NULL");
    HIP_TRY(launch_rng_uniforms(seed, row_offset, n_rows, slot, stream_id, out, (hipStream_t)hip_stream));
    return CSD_OK;
}

}  // extern "C"
