// Block executor: packs weights, owns the per (plan, block) activation store, and runs the
// stage list of one denoising block over the patch batch with optional patch-level cache
// reuse ("Patch-aware Caching Strategy": mask per patch before the block, pixel-wise
// operators recompute only unmasked patches, context operators take the cached operand of
// masked patches, masked outputs are replaced by the cache, the cache is then refreshed).
//
// Reuse without copies: the cached operand tensors ARE the working buffers.  A context
// operator's producer writes only the computed patches into the slot, so after the write the
// slot holds "fresh on computed, previous step on reused" — exactly the operand the
// consumer needs and exactly the refreshed cache for the next step.
#include "kernels.h"

#include <algorithm>
#include <new>
#include <string.h>

using namespace pserve;

namespace pserve {
static int g_kernel_mode = 0;

// ---- optional per-kernel event timing ---------------------------------------------------------
struct ProfRecord { const char* name; hipEvent_t start, stop; };
struct Profiler {
    bool on = false;
    char only[32] = {0};                 // when not empty: the one kernel label that is timed
    int every = 1;                       // time the kernels of every n-th pserve_block_forward call only
    long tick = -1;                      // index of the current pserve_block_forward call
    std::vector<ProfRecord> recs;
    std::vector<hipEvent_t> pool;
    hipEvent_t get() {
        if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
};
static Profiler g_prof;
struct ProfScope {
    hipStream_t st;
    hipEvent_t stop = nullptr;
    ProfScope(const char* name, hipStream_t s) : st(s) {
        if (!g_prof.on || (g_prof.only[0] && strcmp(g_prof.only, name) != 0)) return;
        if (g_prof.every > 1 && g_prof.tick % g_prof.every != 0) return;
        hipEvent_t start = g_prof.get();
        stop = g_prof.get();
        if (!start || !stop) { stop = nullptr; return; }
        (void)hipEventRecord(start, st);
        g_prof.recs.push_back({name, start, stop});
    }
    ~ProfScope() {
        if (stop) (void)hipEventRecord(stop, st);
    }
};

struct StageWeights {
    void* gn_g[2] = {};      // raw copies, block dtype
    void* gn_b[2] = {};
    void* w[5] = {};         // packed [taps][N][K]  (MMDIT: 0 qkv, 1 out, 3 mlp in, 4 mlp out)
    float* b[5] = {};        // packed biases (fp32)
    void* wt = nullptr;      // RES2T: time projection [temb_dim][C], block dtype (raw copy)
    float* bt = nullptr;     // RES2T: its bias (fp32)
};

// ---- small kernels ---------------------------------------------------------------------------------
// Time embedding of the RES2T stages: e[s][c] = bt[c] + sum_k SiLU(temb[perm[s]][k]) * wt[k][c] for request slot s
// (sorted order).  One block of 1024 threads per (slot, 64 channels): 16 thread groups take every 16th k (the sum is a
// chain of dependent loads otherwise: 94 us for 1280 terms), eight loads in flight each; SiLU(temb) is staged once in
// LDS; the 16 partial sums are added in a fixed order.  fp32 accumulation.
constexpr int TEMB_KG = 16;
template <typename T>
__global__ void __launch_bounds__(1024)
temb_proj_kernel(const T* __restrict__ temb, const T* __restrict__ wt, const float* __restrict__ bt,
                 const int32_t* __restrict__ perm, int32_t D, int32_t C, float* __restrict__ e) {
    extern __shared__ float s_t[];                  // [D] SiLU(temb), then [TEMB_KG][64] partial sums
    float* s_part = s_t + D;
    const int s = blockIdx.x;
    const T* tv = temb + (int64_t)perm[s] * D;
    auto as_f = [](T v) -> float {
        if constexpr (sizeof(T) == 2) return __uint_as_float((uint32_t)v << 16);
        else return v;
    };
    for (int k = threadIdx.x; k < D; k += blockDim.x) {
        const float v = as_f(tv[k]);
        s_t[k] = v / (1.f + __expf(-v));
    }
    __syncthreads();
    const int cl = threadIdx.x & 63, kg = threadIdx.x >> 6;
    const int c = min(blockIdx.y * 64 + cl, C - 1);
    float acc = 0.f;
    int k = kg;
    for (; k + 7 * TEMB_KG < D; k += 8 * TEMB_KG) {
        float w[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) w[u] = as_f(wt[(int64_t)(k + u * TEMB_KG) * C + c]);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc = fmaf(s_t[k + u * TEMB_KG], w[u], acc);
    }
    for (; k < D; k += TEMB_KG) acc = fmaf(s_t[k], as_f(wt[(int64_t)k * C + c]), acc);
    s_part[kg * 64 + cl] = acc;
    __syncthreads();
    if (kg == 0 && blockIdx.y * 64 + cl < C) {
        float sum = bt[c];
        for (int g = 0; g < TEMB_KG; ++g) sum += s_part[g * 64 + cl];
        e[(int64_t)s * C + c] = sum;
    }
}

// The same for wide outputs (adaLN modulation: three or six rows of C per request): one block per (pair of request
// slots, 2 * LPR channels); LPR lanes x two adjacent channels (4-byte loads of bf16 pairs) cover the channels, the
// 1024 / LPR thread groups take every (1024 / LPR)-th k.  The weights are read once per pair of slots, and the launch
// picks LPR = 32 or 64 so that the grid is close to one block per CU (the one-slot form ran more than a round of
// 1,024-thread blocks: 24 -> 15 us at 4 x 4,608 x 1536, 29 -> 18 us at 4 x 9,216 x 1536).
template <typename T, int LPR>
__global__ void __launch_bounds__(1024)
temb_proj_wide_kernel(const T* __restrict__ temb, const T* __restrict__ wt, const float* __restrict__ bt,
                      const int32_t* __restrict__ perm, int32_t n, int32_t D, int32_t C, float* __restrict__ e) {
    constexpr int TEMB_WKG = 1024 / LPR, CPB = 2 * LPR;     // k groups, channels per block
    extern __shared__ float s_t[];                  // [2][D] SiLU(temb) of the two slots, then [TEMB_WKG][2][CPB] partial sums
    float* s_part = s_t + 2 * D;
    const int s0 = 2 * blockIdx.x, s1 = min(s0 + 1, n - 1);
    auto as_f = [](T v) -> float {
        if constexpr (sizeof(T) == 2) return __uint_as_float((uint32_t)v << 16);
        else return v;
    };
    for (int k = threadIdx.x; k < 2 * D; k += blockDim.x) {
        const int which = k >= D, kk = k - which * D;
        const float v = as_f(temb[(int64_t)perm[which ? s1 : s0] * D + kk]);
        s_t[k] = v / (1.f + __expf(-v));
    }
    __syncthreads();
    const int cl = threadIdx.x % LPR, kg = threadIdx.x / LPR;
    const int c = min(blockIdx.y * CPB + 2 * cl, C - 2);       // C is even (checked by the launch)
    float acc[2][2] = {};
    auto ld2 = [&](int k, float (&w)[2]) {
        if constexpr (sizeof(T) == 2) {
            const uint32_t r = *reinterpret_cast<const uint32_t*>(wt + (int64_t)k * C + c);
            w[0] = __uint_as_float(r << 16);
            w[1] = __uint_as_float(r & 0xFFFF0000u);
        } else {
            const float2 r = *reinterpret_cast<const float2*>(wt + (int64_t)k * C + c);
            w[0] = r.x;
            w[1] = r.y;
        }
    };
    int k = kg;
    for (; k + 7 * TEMB_WKG < D; k += 8 * TEMB_WKG) {
        float w[8][2];
#pragma unroll
        for (int u = 0; u < 8; ++u) ld2(k + u * TEMB_WKG, w[u]);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float t0 = s_t[k + u * TEMB_WKG], t1 = s_t[D + k + u * TEMB_WKG];
            acc[0][0] = fmaf(t0, w[u][0], acc[0][0]);
            acc[0][1] = fmaf(t0, w[u][1], acc[0][1]);
            acc[1][0] = fmaf(t1, w[u][0], acc[1][0]);
            acc[1][1] = fmaf(t1, w[u][1], acc[1][1]);
        }
    }
    for (; k < D; k += TEMB_WKG) {
        float w[2];
        ld2(k, w);
        const float t0 = s_t[k], t1 = s_t[D + k];
        acc[0][0] = fmaf(t0, w[0], acc[0][0]);
        acc[0][1] = fmaf(t0, w[1], acc[0][1]);
        acc[1][0] = fmaf(t1, w[0], acc[1][0]);
        acc[1][1] = fmaf(t1, w[1], acc[1][1]);
    }
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int h = 0; h < 2; ++h) s_part[(kg * 2 + q) * CPB + 2 * cl + h] = acc[q][h];
    __syncthreads();
    // thread (q, channel): the partial sums of the k groups in a fixed order
    if (threadIdx.x < 2 * CPB) {
        const int q = threadIdx.x / CPB, ch = threadIdx.x % CPB;
        const int cc = blockIdx.y * CPB + ch;
        const int s = q ? s0 + 1 : s0;
        if (cc < C && s < n) {
            float sum = bt[cc];
            for (int g = 0; g < TEMB_WKG; ++g) sum += s_part[(g * 2 + q) * CPB + ch];
            e[(int64_t)s * C + cc] = sum;
        }
    }
}

// Ordered compaction of the patches with mask == 0.
__global__ void compact_mask_kernel(const uint8_t* __restrict__ mask, int32_t P, int32_t* __restrict__ active,
                                    int32_t* __restrict__ count) {
    __shared__ int32_t s_scan[1024];
    __shared__ int32_t carry;
    const int tid = threadIdx.x;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < P; base += 1024) {
        const int p = base + tid;
        const int32_t f = (p < P && mask[p] == 0) ? 1 : 0;
        s_scan[tid] = f;
        __syncthreads();
        for (int off = 1; off < 1024; off <<= 1) {
            int32_t v = 0;
            if (tid >= off) v = s_scan[tid - off];
            __syncthreads();
            s_scan[tid] += v;
            __syncthreads();
        }
        if (f) active[carry + s_scan[tid] - 1] = p;
        __syncthreads();
        if (tid == 1023) carry += s_scan[tid];
        __syncthreads();
    }
    if (tid == 0) *count = carry;
}

// Copy whole patches ([S][C] rows) between token-major tensors, 16 bytes per thread.
// which: 0 = all patches, 1 = patches with mask == 0 (computed), 2 = patches with mask == 1 (reused)
__global__ void copy_patches_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t vec_per_patch,
                                    const uint8_t* __restrict__ mask, int which) {
    const int p = blockIdx.x;
    if (which && mask) {
        const bool reused = mask[p] != 0;
        if ((which == 1) == reused) return;
    } else if (which == 2) {
        return;
    }
    const uint4* s = src + (int64_t)p * vec_per_patch;
    uint4* d = dst + (int64_t)p * vec_per_patch;
    for (int64_t i = blockIdx.y * blockDim.x + threadIdx.x; i < vec_per_patch; i += (int64_t)gridDim.y * blockDim.x) d[i] = s[i];
}

// Coalesced insert of the Common Set into another batch's cache ("Batching Patches in Cache"): new patch p takes the
// rows of old patch src_of[p] (token-major slot, 16 bytes per thread); patches with src_of[p] < 0 are left alone.
__global__ void gather_patches_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t vec_per_patch,
                                      const int32_t* __restrict__ src_of) {
    const int p = blockIdx.x, q = src_of[p];
    if (q < 0) return;
    const uint4* s = src + (int64_t)q * vec_per_patch;
    uint4* d = dst + (int64_t)p * vec_per_patch;
    for (int64_t i = blockIdx.y * blockDim.x + threadIdx.x; i < vec_per_patch; i += (int64_t)gridDim.y * blockDim.x) d[i] = s[i];
}
// The same for a channel-major slot (V^T [C][T]): per channel row, the S tokens of the patch are contiguous.
template <typename T>
__global__ void gather_patch_cols_kernel(const T* __restrict__ src, T* __restrict__ dst, int64_t T_old, int64_t T_new,
                                         int32_t S, int32_t C, const int32_t* __restrict__ src_of) {
    const int p = blockIdx.x, q = src_of[p];
    if (q < 0) return;
    for (int64_t i = blockIdx.y * blockDim.x + threadIdx.x; i < (int64_t)S * C; i += (int64_t)gridDim.y * blockDim.x) {
        const int64_t c = i / S, t = i - c * S;
        dst[c * T_new + (int64_t)p * S + t] = src[c * T_old + (int64_t)q * S + t];
    }
}
__global__ void patch_valid_kernel(const int32_t* __restrict__ src_of, int32_t P, uint8_t* __restrict__ valid) {
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p < P) valid[p] = src_of[p] >= 0 ? 1 : 0;
}

// dst[c][t] = src[t][c] (or the reverse), used by the cache load/read hooks for the transposed V slot
template <typename T>
__global__ void transpose_tc_kernel(const T* __restrict__ src, T* __restrict__ dst, int64_t Tn, int32_t C, int to_ct) {
    __shared__ T tile[32][33];
    const int64_t t0 = (int64_t)blockIdx.x * 32;
    const int c0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    if (to_ct) {
        for (int r = ty; r < 32; r += 8)
            if (t0 + r < Tn && c0 + tx < C) tile[r][tx] = src[(t0 + r) * C + c0 + tx];
        __syncthreads();
        for (int r = ty; r < 32; r += 8)
            if (c0 + r < C && t0 + tx < Tn) dst[(int64_t)(c0 + r) * Tn + t0 + tx] = tile[tx][r];
    } else {
        for (int r = ty; r < 32; r += 8)
            if (c0 + r < C && t0 + tx < Tn) tile[r][tx] = src[(int64_t)(c0 + r) * Tn + t0 + tx];
        __syncthreads();
        for (int r = ty; r < 32; r += 8)
            if (t0 + r < Tn && c0 + tx < C) dst[(t0 + r) * C + c0 + tx] = tile[tx][r];
    }
}
}  // namespace pserve

struct pserve_block_s {
    pserve_block_desc desc;
    StageWeights sw[PSERVE_MAX_STAGES];
    StageWeights sw_txt[PSERVE_MAX_STAGES];   // MMDIT: the text stream's weights (sw holds the image stream's)
    DevicePool pool;
};

struct pserve_cache_s {
    const pserve_plan_t* plan = nullptr;
    const pserve_block_t* block = nullptr;
    bool with_slots = false, filled = false, v_transposed = false;
    int32_t nsplit = 1, cross_ld = 0;
    void* ping[2] = {};                       // [T][C] stage outputs
    void* apad = nullptr;                     // [P][ph+2][pw+2][C]
    float* partial = nullptr;
    float* scale_shift = nullptr;
    // per-channel moments of the block input left behind by pserve_split_stats: [P][in_nch][C][2]; in_stats_x = the x
    // they were taken from (the next forward call on that x uses them once instead of a statistics pass)
    float* in_partial = nullptr;
    int32_t in_nch = 0;
    const void* in_stats_x = nullptr;
    void* h1[PSERVE_MAX_STAGES] = {};         // RES2: first convolution output (slot H1)
    void* r[PSERVE_MAX_STAGES] = {};          // SATTN: stage input (slot R), only with slots
    void* k[PSERVE_MAX_STAGES] = {};          // SATTN: keys (slot K)
    void* v[PSERVE_MAX_STAGES] = {};          // SATTN: values (slot V; [C][T] when v_transposed)
    void* q = nullptr;                        // [T][C] scaled queries
    void* o = nullptr;                        // [T][C] attention output
    void* u = nullptr;                        // [T][C] normalised tokens
    void* kc = nullptr;                       // [n*cross_ld][C] text keys
    void* vc = nullptr;                       // [n*cross_ld][C] text values
    void* hidden = nullptr;                   // [T][F]
    void* yslot = nullptr;                    // [T][C] block output of the previous step (slot Y)
    float* temb_e[PSERVE_MAX_STAGES] = {};    // RES2T: [n][C] projected time embedding per request slot
    float* temb_e2[PSERVE_MAX_STAGES] = {};   // MMDIT: [n][6C] modulation of the text stream (temb_e: image stream)
    int32_t* stream_list[2] = {};             // MMDIT: image patches / text patches of the joint plan (ascending)
    int32_t* stream_count = nullptr;          // [2] their numbers
    int32_t* active = nullptr;
    int32_t* count = nullptr;
    int32_t* act_off = nullptr;               // [n+1] attention: computed patches before slot s
    int32_t* tile_off = nullptr;              // [n+1] attention: query tiles before slot s
    int32_t max_tiles = 0;
    int32_t att_qt = 2;                       // query tile of the MFMA attention: 128 * att_qt rows
    bool tiles_unmasked = false;              // act_off / tile_off hold the tiling of a call without mask
    // The text key / value projection of the one cross-attention stage depends on ctx only: it runs on a stream of
    // its own (default priority) beside the stages before it, forked and joined with events.
    hipStream_t side = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    hipEvent_t ev_temb[PSERVE_MAX_STAGES] = {};   // projection of the per-request vector of stage s is done (side stream)
    hipEvent_t ev_txt[4] = {};                    // joint block: fork / join of the text stream's kernels (side stream)
    bool side_temb = false;                       // the projections run on the side stream (else inline, at their stage)
    int side_stage = -1;
    DevicePool pool;
    ~pserve_cache_s() {
        if (ev_fork) (void)hipEventDestroy(ev_fork);
        if (ev_join) (void)hipEventDestroy(ev_join);
        for (hipEvent_t e : ev_temb) if (e) (void)hipEventDestroy(e);
        for (hipEvent_t e : ev_txt) if (e) (void)hipEventDestroy(e);
        if (side) (void)hipStreamDestroy(side);
    }
};

static bool has_stage(const pserve_block_desc& d, int kind) {
    for (int i = 0; i < d.n_stages; ++i)
        if (d.stages[i] == kind) return true;
    return false;
}
// stage families: the L-kinds are the token stages with a LayerNorm in front
static bool is_sattn(int k) { return k == PSERVE_SATTN || k == PSERVE_LSATTN || k == PSERVE_ASATTN || k == PSERVE_MMDIT; }
static bool is_xattn(int k) { return k == PSERVE_XATTN || k == PSERVE_LXATTN; }
static bool is_ffn(int k) { return k == PSERVE_FFN || k == PSERVE_LFFN; }
static bool is_res2(int k) { return k == PSERVE_RES2 || k == PSERVE_RES2T; }
static bool has_ln(int k) { return k == PSERVE_LSATTN || k == PSERVE_LXATTN || k == PSERVE_LFFN || k == PSERVE_ASATTN || k == PSERVE_AMLP; }
static bool has_mod(int k) { return k == PSERVE_ASATTN || k == PSERVE_AMLP; }
static bool needs_temb(int k) { return k == PSERVE_RES2T || has_mod(k) || k == PSERVE_MMDIT; }
template <typename F> static bool any_stage(const pserve_block_desc& d, F f) {
    for (int s = 0; s < d.n_stages; ++s) if (f(d.stages[s])) return true;
    return false;
}

static int dup_param(DevicePool& pool, const void* src, size_t bytes, void** dst, hipStream_t st) {
    PS_TRY(pool.alloc(dst, bytes));
    PS_CHECK_HIP(hipMemcpyAsync(*dst, src, bytes, hipMemcpyDeviceToDevice, st));
    return PSERVE_OK;
}

extern "C" {

int pserve_set_kernel_mode(int mode) {
    PS_REQUIRE(mode >= 0 && mode <= 2, "pserve_set_kernel_mode: mode must be 0, 1 or 2");
    g_kernel_mode = mode;
    return PSERVE_OK;
}

int pserve_profile_enable(int on) {
    g_prof.on = on != 0;
    return PSERVE_OK;
}

int pserve_profile_sample(int every) {
    PS_REQUIRE(every >= 1, "pserve_profile_sample: every must be at least 1");
    g_prof.every = every;
    g_prof.tick = -1;
    return PSERVE_OK;
}

int pserve_profile_select(const char* label) {
    memset(g_prof.only, 0, sizeof(g_prof.only));
    if (label) {
        PS_REQUIRE(strlen(label) < sizeof(g_prof.only), "pserve_profile_select: label too long");
        strcpy(g_prof.only, label);
    }
    return PSERVE_OK;
}

static int profile_read_impl(pserve_prof_entry* out, int32_t max, int32_t* count) {
    PS_REQUIRE(out && count && max > 0, "pserve_profile_read: bad arguments");
    int n = 0;
    for (const ProfRecord& r : g_prof.recs) {
        PS_CHECK_HIP(hipEventSynchronize(r.stop));
        float ms = 0.f;
        PS_CHECK_HIP(hipEventElapsedTime(&ms, r.start, r.stop));
        int k = 0;
        while (k < n && strncmp(out[k].name, r.name, sizeof(out[k].name)) != 0) ++k;
        if (k == n) {
            if (n == max) continue;
            memset(&out[n], 0, sizeof(out[n]));
            strncpy(out[n].name, r.name, sizeof(out[n].name) - 1);
            ++n;
        }
        out[k].calls += 1;
        out[k].total_ms += ms;
    }
    for (const ProfRecord& r : g_prof.recs) { g_prof.pool.push_back(r.start); g_prof.pool.push_back(r.stop); }
    g_prof.recs.clear();
    *count = n;
    return PSERVE_OK;
}

int pserve_profile_read(pserve_prof_entry* out, int32_t max, int32_t* count) {
    return guarded("pserve_profile_read", [&] { return profile_read_impl(out, max, count); });
}

static int block_create_impl(const pserve_block_desc* desc, const pserve_block_params* params, void* stream, pserve_block_t** out) {
    PS_REQUIRE(out, "pserve_block_create: out is NULL");
    *out = nullptr;
    PS_REQUIRE(desc && params, "pserve_block_create: NULL argument");
    const pserve_block_desc& d = *desc;
    PS_REQUIRE(d.n_stages > 0 && d.n_stages <= PSERVE_MAX_STAGES, "pserve_block_create: n_stages=%d out of range", d.n_stages);
    PS_REQUIRE(d.dtype == PSERVE_F32 || d.dtype == PSERVE_BF16, "pserve_block_create: unknown dtype %d", d.dtype);
    PS_REQUIRE(d.C > 0 && d.G > 0 && d.C % d.G == 0, "pserve_block_create: C=%d must be a positive multiple of G=%d", d.C, d.G);
    PS_REQUIRE(d.C % (d.dtype == PSERVE_BF16 ? 8 : 4) == 0, "pserve_block_create: C=%d must be a multiple of 16 bytes", d.C);
    PS_REQUIRE(d.eps >= 0.f, "pserve_block_create: negative eps");
    static const int nparams[13] = {0, 4, 8, 7, 5, 4, 7, 7, 6, 10, 7, 6, 22};
    for (int s = 0; s < d.n_stages; ++s) {
        const int kind = d.stages[s];
        PS_REQUIRE(kind >= PSERVE_RES1 && kind <= PSERVE_MMDIT, "pserve_block_create: stage %d has unknown kind %d", s, kind);
        PS_REQUIRE((kind == PSERVE_MMDIT) == (d.stages[0] == PSERVE_MMDIT), "pserve_block_create: joint blocks hold PSERVE_MMDIT stages only");
        for (int k = 0; k < nparams[kind]; ++k) PS_REQUIRE(params->p[s][k], "pserve_block_create: stage %d parameter %d is NULL", s, k);
        if (is_sattn(kind) || is_xattn(kind))
            PS_REQUIRE(d.heads > 0 && d.C % d.heads == 0 && d.C / d.heads <= 128,
                       "pserve_block_create: heads=%d must divide C=%d with head dim <= 128", d.heads, d.C);
        if (needs_temb(kind))
            PS_REQUIRE(d.temb_dim > 0 && d.temb_dim <= 8192, "pserve_block_create: stage %d needs temb_dim in 1..8192 (got %d)", s, d.temb_dim);
        if (kind == PSERVE_AMLP || kind == PSERVE_MMDIT)
            PS_REQUIRE(d.ffn_mult > 0, "pserve_block_create: AMLP / MMDIT need ffn_mult > 0");
        if (is_xattn(kind))
            PS_REQUIRE(d.ctx_len > 0 && d.ctx_dim > 0, "pserve_block_create: XATTN needs ctx_len and ctx_dim");
        if (is_ffn(kind))
            PS_REQUIRE(d.ffn_mult > 0 && (d.ffn_mult * d.C) % GEGLU_GROUP == 0,
                       "pserve_block_create: FFN hidden width %d must be a multiple of %d", d.ffn_mult * d.C, GEGLU_GROUP);
    }
    pserve_block_t* b = new (std::nothrow) pserve_block_t();
    if (!b) { set_error("pserve_block_create: out of host memory"); return PSERVE_ENOMEM; }
    struct Guard { pserve_block_t* p; ~Guard() { delete p; } } guard{b};
    b->desc = d;
    hipStream_t st = (hipStream_t)stream;
    const size_t es = dtype_size(d.dtype);
    const int C = d.C;
    for (int s = 0; s < d.n_stages; ++s) {
        StageWeights& w = b->sw[s];
        const void* const* p = params->p[s];
        if (has_mod(d.stages[s])) {                                            // wm bm, then the sub-layer's own parameters
            PS_TRY(dup_param(b->pool, p[0], es * d.temb_dim * 3 * C, &w.wt, st));
            PS_TRY(b->pool.alloc_t(&w.bt, 3 * C));
            PS_TRY(pack_bias(p[1], w.bt, 3 * C, d.dtype, st));
            p += 2;
        }
        if (d.stages[s] == PSERVE_LXATTN || d.stages[s] == PSERVE_LFFN) {     // ln_g ln_b, then the parameters of the plain kind
            PS_TRY(dup_param(b->pool, p[0], es * C, &w.gn_g[0], st));
            PS_TRY(dup_param(b->pool, p[1], es * C, &w.gn_b[0], st));
            p += 2;
        }
        switch (d.stages[s]) {
        case PSERVE_RES1:
        case PSERVE_RES2:
        case PSERVE_RES2T: {
            const int convs = d.stages[s] == PSERVE_RES1 ? 1 : 2;
            if (d.stages[s] == PSERVE_RES2T) {
                PS_TRY(dup_param(b->pool, p[8], es * d.temb_dim * C, &w.wt, st));
                PS_TRY(b->pool.alloc_t(&w.bt, C));
                PS_TRY(pack_bias(p[9], w.bt, C, d.dtype, st));
            }
            for (int c = 0; c < convs; ++c) {
                PS_TRY(dup_param(b->pool, p[4 * c + 0], es * C, &w.gn_g[c], st));
                PS_TRY(dup_param(b->pool, p[4 * c + 1], es * C, &w.gn_b[c], st));
                PS_TRY(b->pool.alloc(&w.w[c], es * 9 * C * C));
                PS_TRY(pack_conv(p[4 * c + 2], w.w[c], C, C, d.dtype, st));
                PS_TRY(b->pool.alloc_t(&w.b[c], C));
                PS_TRY(pack_bias(p[4 * c + 3], w.b[c], C, d.dtype, st));
            }
            break;
        }
        case PSERVE_SATTN:
        case PSERVE_LSATTN:                                                    // norm parameters first in both kinds
        case PSERVE_ASATTN: {                                                  // (p already points behind wm bm)
            const int o = d.stages[s] == PSERVE_ASATTN ? 0 : 2;
            if (o) {
                PS_TRY(dup_param(b->pool, p[0], es * C, &w.gn_g[0], st));
                PS_TRY(dup_param(b->pool, p[1], es * C, &w.gn_b[0], st));
            }
            PS_TRY(b->pool.alloc(&w.w[0], es * 3 * C * C));                       // fused [Wq | Wk | Wv]
            for (int k = 0; k < 3; ++k) PS_TRY(pack_linear(p[o + k], w.w[0], C, C, k * C, d.dtype, st));
            PS_TRY(b->pool.alloc(&w.w[1], es * C * C));
            PS_TRY(pack_linear(p[o + 3], w.w[1], C, C, 0, d.dtype, st));
            PS_TRY(b->pool.alloc_t(&w.b[1], C));
            PS_TRY(pack_bias(p[o + 4], w.b[1], C, d.dtype, st));
            break;
        }
        case PSERVE_MMDIT: {
            const int F = d.ffn_mult * C;
            for (int x = 0; x < 2; ++x) {                                         // image stream, text stream
                StageWeights& v = x == 0 ? b->sw[s] : b->sw_txt[s];
                const void* const* q = p + 11 * x;
                PS_TRY(dup_param(b->pool, q[0], es * d.temb_dim * 6 * C, &v.wt, st));
                PS_TRY(b->pool.alloc_t(&v.bt, 6 * C));
                PS_TRY(pack_bias(q[1], v.bt, 6 * C, d.dtype, st));
                PS_TRY(b->pool.alloc(&v.w[0], es * 3 * C * C));
                for (int k = 0; k < 3; ++k) PS_TRY(pack_linear(q[2 + k], v.w[0], C, C, k * C, d.dtype, st));
                PS_TRY(b->pool.alloc(&v.w[1], es * C * C));
                PS_TRY(pack_linear(q[5], v.w[1], C, C, 0, d.dtype, st));
                PS_TRY(b->pool.alloc_t(&v.b[1], C));
                PS_TRY(pack_bias(q[6], v.b[1], C, d.dtype, st));
                PS_TRY(b->pool.alloc(&v.w[3], es * F * C));
                PS_TRY(pack_linear(q[7], v.w[3], C, F, 0, d.dtype, st));
                PS_TRY(b->pool.alloc_t(&v.b[3], F));
                PS_TRY(pack_bias(q[8], v.b[3], F, d.dtype, st));
                PS_TRY(b->pool.alloc(&v.w[4], es * C * F));
                PS_TRY(pack_linear(q[9], v.w[4], F, C, 0, d.dtype, st));
                PS_TRY(b->pool.alloc_t(&v.b[4], C));
                PS_TRY(pack_bias(q[10], v.b[4], C, d.dtype, st));
            }
            break;
        }
        case PSERVE_AMLP: {
            const int F = d.ffn_mult * C;
            PS_TRY(b->pool.alloc(&w.w[0], es * F * C));
            PS_TRY(pack_linear(p[0], w.w[0], C, F, 0, d.dtype, st));
            PS_TRY(b->pool.alloc_t(&w.b[0], F));
            PS_TRY(pack_bias(p[1], w.b[0], F, d.dtype, st));
            PS_TRY(b->pool.alloc(&w.w[1], es * C * F));
            PS_TRY(pack_linear(p[2], w.w[1], F, C, 0, d.dtype, st));
            PS_TRY(b->pool.alloc_t(&w.b[1], C));
            PS_TRY(pack_bias(p[3], w.b[1], C, d.dtype, st));
            break;
        }
        case PSERVE_XATTN:
        case PSERVE_LXATTN: {
            const int D = d.ctx_dim;
            PS_TRY(b->pool.alloc(&w.w[0], es * C * C));
            PS_TRY(pack_linear(p[0], w.w[0], C, C, 0, d.dtype, st));
            PS_TRY(b->pool.alloc(&w.w[2], es * 2 * C * D));                       // fused [Wk | Wv] on the text tokens
            PS_TRY(pack_linear(p[1], w.w[2], D, C, 0, d.dtype, st));
            PS_TRY(pack_linear(p[2], w.w[2], D, C, C, d.dtype, st));
            PS_TRY(b->pool.alloc(&w.w[1], es * C * C));
            PS_TRY(pack_linear(p[3], w.w[1], C, C, 0, d.dtype, st));
            PS_TRY(b->pool.alloc_t(&w.b[1], C));
            PS_TRY(pack_bias(p[4], w.b[1], C, d.dtype, st));
            break;
        }
        case PSERVE_FFN:
        case PSERVE_LFFN: {
            const int F = d.ffn_mult * C;
            PS_TRY(b->pool.alloc(&w.w[0], es * 2 * F * C));
            PS_TRY(b->pool.alloc_t(&w.b[0], 2 * F));
            PS_TRY(pack_geglu(p[0], p[1], w.w[0], w.b[0], C, F, d.dtype, st));
            PS_TRY(b->pool.alloc(&w.w[1], es * C * F));
            PS_TRY(pack_linear(p[2], w.w[1], F, C, 0, d.dtype, st));
            PS_TRY(b->pool.alloc_t(&w.b[1], C));
            PS_TRY(pack_bias(p[3], w.b[1], C, d.dtype, st));
            break;
        }
        }
    }
    PS_CHECK_HIP(hipStreamSynchronize(st));
    guard.p = nullptr;
    *out = b;
    return PSERVE_OK;
}

int pserve_block_create(const pserve_block_desc* desc, const pserve_block_params* params, void* stream, pserve_block_t** out) {
    return guarded("pserve_block_create", [&] { return block_create_impl(desc, params, stream, out); });
}

void pserve_block_free(pserve_block_t* block) { delete block; }

static int cache_create_impl(const pserve_plan_t* plan, const pserve_block_t* block, int with_slots, pserve_cache_t** out) {
    PS_REQUIRE(out, "pserve_cache_create: out is NULL");
    *out = nullptr;
    PS_REQUIRE(plan && block, "pserve_cache_create: NULL argument");
    const pserve_block_desc& d = block->desc;
    if (with_slots)
        for (int s = 1; s < d.n_stages; ++s)
            PS_REQUIRE(d.stages[s] != PSERVE_RES1 && !is_res2(d.stages[s]),
                       "pserve_cache_create: patch reuse needs residual-convolution stages at position 0 only "
                       "(their input statistics and halos must be fresh on every patch)");
    const bool joint = has_stage(d, PSERVE_MMDIT);
    PS_REQUIRE(joint == (plan->text_len > 0), "pserve_cache_create: PSERVE_MMDIT stages need a joint plan (pserve_plan_text), other stages a plain one");
    PS_REQUIRE(!(joint && with_slots), "pserve_cache_create: joint blocks have no cache slots");
    pserve_cache_t* c = new (std::nothrow) pserve_cache_t();
    if (!c) { set_error("pserve_cache_create: out of host memory"); return PSERVE_ENOMEM; }
    struct Guard { pserve_cache_t* p; ~Guard() { delete p; } } guard{c};
    c->plan = plan;
    c->block = block;
    c->with_slots = with_slots != 0;
    const size_t es = dtype_size(d.dtype);
    const size_t TC = (size_t)plan->T * d.C * es;
    const int head_dim = d.heads > 0 ? d.C / d.heads : 0;
    c->v_transposed = d.dtype == PSERVE_BF16 && head_dim == 64 && g_kernel_mode != 1;
    c->nsplit = (int)std::max<int64_t>(1, std::min<int64_t>(cdiv(768, plan->P), std::max(1, plan->S / 32)));
    PS_TRY(c->pool.alloc(&c->ping[0], TC));
    PS_TRY(c->pool.alloc(&c->ping[1], TC));
    const bool conv = has_stage(d, PSERVE_RES1) || any_stage(d, is_res2);
    const bool sattn = any_stage(d, is_sattn), xattn = any_stage(d, is_xattn);
    const bool ffn = any_stage(d, is_ffn) || has_stage(d, PSERVE_AMLP) || joint;
    const bool gn_sattn = has_stage(d, PSERVE_SATTN);
    if (conv) PS_TRY(c->pool.alloc(&c->apad, (size_t)plan->P * (plan->ph + 2) * (plan->pw + 2) * d.C * es));
    if (conv || gn_sattn) {
        PS_TRY(c->pool.alloc_t(&c->partial, (size_t)plan->P * std::max<int64_t>(c->nsplit, plan->S / 64) * d.G * 2));
        PS_TRY(c->pool.alloc_t(&c->scale_shift, (size_t)plan->n * d.C * 2));
        // token chunks per patch of the split pass that also takes the input's moments: enough blocks to fill the
        // chip (x C / 64 channel slabs), a divisor of the patch's 32-token tiles
        if (d.dtype == PSERVE_BF16 && plan->S % 32 == 0 && d.C % 64 == 0) {
            int nch = 8;
            while (nch > 1 && (plan->S / 32) % nch != 0) nch >>= 1;
            c->in_nch = nch;
            PS_TRY(c->pool.alloc_t(&c->in_partial, (size_t)plan->P * nch * d.C * 2));
        }
    }
    for (int s = 0; s < d.n_stages; ++s) {
        if (is_res2(d.stages[s])) PS_TRY(c->pool.alloc(&c->h1[s], TC));
        if (d.stages[s] == PSERVE_RES2T) PS_TRY(c->pool.alloc_t(&c->temb_e[s], (size_t)plan->n * d.C));
        if (has_mod(d.stages[s])) PS_TRY(c->pool.alloc_t(&c->temb_e[s], (size_t)plan->n * 3 * d.C));
        if (d.stages[s] == PSERVE_MMDIT) {
            PS_TRY(c->pool.alloc_t(&c->temb_e[s], (size_t)plan->n * 6 * d.C));
            PS_TRY(c->pool.alloc_t(&c->temb_e2[s], (size_t)plan->n * 6 * d.C));
        }
        if (is_sattn(d.stages[s])) {
            if (with_slots && d.stages[s] == PSERVE_SATTN) PS_TRY(c->pool.alloc(&c->r[s], TC));
            PS_TRY(c->pool.alloc(&c->k[s], TC));
            PS_TRY(c->pool.alloc(&c->v[s], TC));
        }
    }
    if (sattn || xattn) {
        PS_TRY(c->pool.alloc(&c->q, TC));
        PS_TRY(c->pool.alloc(&c->o, TC));
    }
    if (sattn || any_stage(d, has_ln)) PS_TRY(c->pool.alloc(&c->u, TC));     // normalised stage input
    if (xattn) {
        // text keys / values: rows padded to a multiple of 8 per request and zero-filled once, so that the
        // padding rows (never written) contribute exact zeros; values transposed like the self-attention V
        c->cross_ld = c->v_transposed ? (d.ctx_len + 7) / 8 * 8 : d.ctx_len;
        const size_t bytes = (size_t)plan->n * c->cross_ld * d.C * es;
        PS_TRY(c->pool.alloc(&c->kc, bytes));
        PS_TRY(c->pool.alloc(&c->vc, bytes));
        PS_CHECK_HIP(hipMemset(c->kc, 0, bytes));
        PS_CHECK_HIP(hipMemset(c->vc, 0, bytes));
    }
    if (sattn || xattn) {
        PS_TRY(c->pool.alloc_t(&c->act_off, (size_t)plan->n + 1));
        PS_TRY(c->pool.alloc_t(&c->tile_off, (size_t)plan->n + 1));
        // The software-pipelined kernel (256-row query tile) as soon as its blocks cover the chip once (256 CUs): with
        // 520 blocks (8 latents of 32^2 / 48^2, 10 heads) it ran in 82 us against 99 us for the 128-row kernel with
        // twice the blocks.  Below that the smaller tile, which gives twice as many blocks to spread.
        c->att_qt = attention_max_tiles(plan, 2) * (int64_t)d.heads < 256 ? 1 : 2;
        c->max_tiles = attention_max_tiles(plan, c->att_qt);
    }
    if (ffn) PS_TRY(c->pool.alloc(&c->hidden, (size_t)plan->T * d.ffn_mult * d.C * es));
    if (with_slots) PS_TRY(c->pool.alloc(&c->yslot, TC));
    PS_TRY(c->pool.alloc_t(&c->active, (size_t)plan->P));
    PS_TRY(c->pool.alloc_t(&c->count, 1));
    if (joint) {                                    // the two streams as patch lists
        std::vector<int32_t> lists[2];
        const auto& rc = plan->h_tab[PSERVE_TAB_PATCH_RC];
        for (int p = 0; p < plan->P; ++p) lists[rc[2 * p] < 0 ? 1 : 0].push_back(p);
        const int32_t counts[2] = {(int32_t)lists[0].size(), (int32_t)lists[1].size()};
        PS_TRY(c->pool.alloc_t(&c->stream_count, 2));
        PS_CHECK_HIP(hipMemcpy(c->stream_count, counts, sizeof(counts), hipMemcpyHostToDevice));
        for (int x = 0; x < 2; ++x) {
            PS_TRY(c->pool.alloc_t(&c->stream_list[x], lists[x].size()));
            PS_CHECK_HIP(hipMemcpy(c->stream_list[x], lists[x].data(), sizeof(int32_t) * lists[x].size(), hipMemcpyHostToDevice));
        }
    }
    {
        int n_x = 0, at = -1;
        for (int k = 0; k < d.n_stages; ++k) if (is_xattn(d.stages[k])) { ++n_x; at = k; }
        const bool side_kv = n_x == 1 && at > 0;   // something runs before it: worth a stream of its own
        // The projections of the per-request vector depend on temb only.  A second stream costs a fork and a join
        // (about 10 us of cross-stream waits): it pays for the adaLN projections of a wide block (2 x 20 us hidden at
        // 1536 channels), not for the 5 us time-embedding projection of a 320-channel residual block.
        int64_t macs = 0;
        for (int k = 0; k < d.n_stages; ++k)
            if (needs_temb(d.stages[k]))
                macs += (int64_t)plan->n * d.temb_dim * (d.stages[k] == PSERVE_RES2T ? d.C : d.stages[k] == PSERVE_MMDIT ? 12 * d.C : 3 * d.C);
        c->side_temb = macs >= (int64_t)8 << 20;
        // A joint block runs the text stream's kernels (5 % of the rows, few tiles each: latency bound) on the side stream,
        // beside the image stream's (config 9: the text kernels alone were 19 % of the block).
        if (side_kv || c->side_temb || joint) {
            PS_CHECK_HIP(hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking));
            if (joint)
                for (hipEvent_t& e : c->ev_txt) PS_CHECK_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
            PS_CHECK_HIP(hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming));
            PS_CHECK_HIP(hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming));
            for (int k = 0; k < d.n_stages; ++k)
                if (c->side_temb && needs_temb(d.stages[k]))
                    PS_CHECK_HIP(hipEventCreateWithFlags(&c->ev_temb[k], hipEventDisableTiming));
            if (side_kv) c->side_stage = at;
        }
    }
    guard.p = nullptr;
    *out = c;
    return PSERVE_OK;
}

int pserve_cache_create(const pserve_plan_t* plan, const pserve_block_t* block, int with_slots, pserve_cache_t** out) {
    return guarded("pserve_cache_create", [&] { return cache_create_impl(plan, block, with_slots, out); });
}

void pserve_cache_free(pserve_cache_t* cache) { delete cache; }

static int slot_ptr(const pserve_cache_t* c, int stage, int slot, void** ptr, bool* transposed) {
    PS_REQUIRE(c, "cache slot: cache is NULL");
    PS_REQUIRE(c->with_slots, "cache slot: this cache was created without slots");
    const pserve_block_desc& d = c->block->desc;
    *transposed = false;
    if (slot == PSERVE_SLOT_Y) {
        PS_REQUIRE(stage == -1, "cache slot: the output slot is addressed with stage = -1");
        *ptr = c->yslot;
        return PSERVE_OK;
    }
    PS_REQUIRE(stage >= 0 && stage < d.n_stages, "cache slot: stage %d out of range", stage);
    void* p = nullptr;
    if (slot == PSERVE_SLOT_H1 && is_res2(d.stages[stage])) p = c->h1[stage];
    else if (slot == PSERVE_SLOT_R && d.stages[stage] == PSERVE_SATTN) p = c->r[stage];
    else if (slot == PSERVE_SLOT_K && is_sattn(d.stages[stage])) p = c->k[stage];
    else if (slot == PSERVE_SLOT_V && is_sattn(d.stages[stage])) { p = c->v[stage]; *transposed = c->v_transposed; }
    PS_REQUIRE(p, "cache slot: stage %d has no slot %d", stage, slot);
    *ptr = p;
    return PSERVE_OK;
}

static int slot_copy(const pserve_cache_t* c, void* slot, bool transposed, void* user, bool load, hipStream_t st) {
    const pserve_block_desc& d = c->block->desc;
    const size_t es = dtype_size(d.dtype);
    const int64_t T = c->plan->T;
    if (!transposed) {
        PS_CHECK_HIP(hipMemcpyAsync(load ? slot : user, load ? user : slot, (size_t)T * d.C * es, hipMemcpyDeviceToDevice, st));
        return PSERVE_OK;
    }
    dim3 grid((unsigned)cdiv(T, 32), (unsigned)cdiv(d.C, 32));
    if (d.dtype == PSERVE_BF16)
        transpose_tc_kernel<uint16_t><<<grid, 256, 0, st>>>((const uint16_t*)(load ? user : slot), (uint16_t*)(load ? slot : user), T, d.C, load ? 1 : 0);
    else
        transpose_tc_kernel<float><<<grid, 256, 0, st>>>((const float*)(load ? user : slot), (float*)(load ? slot : user), T, d.C, load ? 1 : 0);
    return check_launch("transpose_tc_kernel");
}

int pserve_cache_load(pserve_cache_t* cache, int stage, int slot, const void* src, void* stream) {
    void* p; bool tr;
    PS_TRY(slot_ptr(cache, stage, slot, &p, &tr));
    PS_REQUIRE(src, "pserve_cache_load: src is NULL");
    PS_TRY(slot_copy(cache, p, tr, (void*)src, true, (hipStream_t)stream));
    cache->filled = true;
    return PSERVE_OK;
}

int pserve_cache_read(const pserve_cache_t* cache, int stage, int slot, void* dst, void* stream) {
    void* p; bool tr;
    PS_TRY(slot_ptr(cache, stage, slot, &p, &tr));
    PS_REQUIRE(dst, "pserve_cache_read: dst is NULL");
    return slot_copy(cache, p, tr, dst, false, (hipStream_t)stream);
}

int pserve_cache_migrate(const pserve_cache_t* old_cache, pserve_cache_t* new_cache, const int32_t* patch_src,
                         uint8_t* valid, void* stream) {
    PS_REQUIRE(old_cache && new_cache && patch_src, "pserve_cache_migrate: NULL argument");
    PS_REQUIRE(old_cache != new_cache, "pserve_cache_migrate: old and new cache are the same object");
    PS_REQUIRE(old_cache->with_slots && new_cache->with_slots, "pserve_cache_migrate: both caches need slots");
    PS_REQUIRE(old_cache->block == new_cache->block, "pserve_cache_migrate: the caches belong to different blocks");
    PS_REQUIRE(old_cache->plan->ph == new_cache->plan->ph && old_cache->plan->pw == new_cache->plan->pw,
               "pserve_cache_migrate: the two plans use different patch sizes");
    PS_REQUIRE(old_cache->v_transposed == new_cache->v_transposed, "pserve_cache_migrate: the caches use different value layouts");
    if (!old_cache->filled) { set_error("pserve_cache_migrate: the old cache was never filled"); return PSERVE_ESTATE; }
    const pserve_block_desc& d = new_cache->block->desc;
    hipStream_t st = (hipStream_t)stream;
    const pserve_plan_t* pn = new_cache->plan;
    const size_t es = dtype_size(d.dtype);
    const int64_t vec_per_patch = (int64_t)pn->S * d.C * es / 16;
    PS_REQUIRE(((int64_t)pn->S * d.C * es) % 16 == 0, "pserve_cache_migrate: a patch must be a multiple of 16 bytes");
    const dim3 grid(pn->P, (unsigned)std::max<int64_t>(1, std::min<int64_t>(cdiv(vec_per_patch, 1024), 64)));
    auto rows = [&](const void* src, void* dst) -> int {
        if (!src || !dst) return PSERVE_OK;
        gather_patches_kernel<<<grid, 256, 0, st>>>((const uint4*)src, (uint4*)dst, vec_per_patch, patch_src);
        return check_launch("gather_patches_kernel");
    };
    for (int s = 0; s < d.n_stages; ++s) {
        PS_TRY(rows(old_cache->h1[s], new_cache->h1[s]));
        PS_TRY(rows(old_cache->r[s], new_cache->r[s]));
        PS_TRY(rows(old_cache->k[s], new_cache->k[s]));
        if (old_cache->v[s] && new_cache->v[s]) {
            if (!new_cache->v_transposed) PS_TRY(rows(old_cache->v[s], new_cache->v[s]));
            else {
                if (d.dtype == PSERVE_BF16)
                    gather_patch_cols_kernel<uint16_t><<<grid, 256, 0, st>>>((const uint16_t*)old_cache->v[s], (uint16_t*)new_cache->v[s],
                                                                             old_cache->plan->T, pn->T, pn->S, d.C, patch_src);
                else
                    gather_patch_cols_kernel<float><<<grid, 256, 0, st>>>((const float*)old_cache->v[s], (float*)new_cache->v[s],
                                                                          old_cache->plan->T, pn->T, pn->S, d.C, patch_src);
                PS_TRY(check_launch("gather_patch_cols_kernel"));
            }
        }
    }
    PS_TRY(rows(old_cache->yslot, new_cache->yslot));
    if (valid) {
        patch_valid_kernel<<<(unsigned)cdiv(pn->P, 256), 256, 0, st>>>(patch_src, pn->P, valid);
        PS_TRY(check_launch("patch_valid_kernel"));
    }
    new_cache->filled = true;
    return PSERVE_OK;
}

int pserve_split_stats(const pserve_plan_t* plan, const void* const* images, int32_t C, int dtype, void* x,
                       pserve_cache_t* cache, void* stream) {
    PS_REQUIRE(plan && images && x && cache, "pserve_split_stats: NULL argument");
    PS_REQUIRE(cache->plan == plan, "pserve_split_stats: cache belongs to another plan");
    cache->in_stats_x = nullptr;
    bool done = false;
    if (cache->in_partial && dtype == PSERVE_BF16 && cache->block->desc.dtype == PSERVE_BF16 && C == cache->block->desc.C &&
        g_kernel_mode != 1)
        PS_TRY(split_with_stats(plan, images, C, x, cache->in_partial, cache->in_nch, (hipStream_t)stream, &done));
    if (!done) return pserve_split(plan, images, C, dtype, x, stream);
    cache->in_stats_x = x;
    return PSERVE_OK;
}

int pserve_block_forward(const pserve_plan_t* plan, const void* x, const void* ctx, const pserve_block_t* block,
                         pserve_cache_t* cache, const uint8_t* reuse_mask, void* y, void* stream) {
    return pserve_block_forward_temb(plan, x, ctx, nullptr, block, cache, reuse_mask, y, stream);
}

int pserve_block_forward_temb(const pserve_plan_t* plan, const void* x, const void* ctx, const void* temb,
                              const pserve_block_t* block, pserve_cache_t* cache, const uint8_t* reuse_mask, void* y,
                              void* stream) {
    PS_REQUIRE(plan && x && block && cache && y, "pserve_block_forward: NULL argument");
    PS_REQUIRE(x != y, "pserve_block_forward: x and y must not alias");
    PS_REQUIRE(cache->plan == plan && cache->block == block, "pserve_block_forward: cache belongs to another plan or block");
    const pserve_block_desc& d = block->desc;
    PS_REQUIRE(ctx || !any_stage(d, is_xattn), "pserve_block_forward: XATTN stage needs ctx");
    PS_REQUIRE(temb || !any_stage(d, needs_temb), "pserve_block_forward: a RES2T / ASATTN / AMLP stage needs temb (pserve_block_forward_temb)");
    if (reuse_mask) {
        if (!cache->with_slots) { set_error("pserve_block_forward: reuse mask given but the cache has no slots"); return PSERVE_ESTATE; }
        if (!cache->filled) { set_error("pserve_block_forward: reuse mask given but the cache was never filled"); return PSERVE_ESTATE; }
    }
    hipStream_t st = (hipStream_t)stream;
    ++g_prof.tick;
    const int dt = d.dtype, C = d.C;
    // moments of this x taken while it was split (single use: later calls on the buffer may see other contents)
    const bool in_stats = cache->in_stats_x == x && cache->in_partial;
    cache->in_stats_x = nullptr;
    const int mode = g_kernel_mode == 1 ? 1 : 0;    // kernels: fastest available / plain reference
    const bool push = g_kernel_mode == 0;           // edge stitching fused into the normalisation / separate gather
    const size_t es = dtype_size(dt);
    PatchGeom gm;
    gm.P = plan->P; gm.S = plan->S; gm.ph = plan->ph; gm.pw = plan->pw;
    gm.ppw = plan->pw + 2; gm.pS = (plan->ph + 2) * (plan->pw + 2);
    const int32_t* request_offset = plan->d_tab[PSERVE_TAB_REQUEST_OFFSET];
    const int32_t* owner = plan->d_tab[PSERVE_TAB_PATCH_OWNER];
    const int64_t T = plan->T;
    const int64_t vec_per_patch = (int64_t)plan->S * C * es / 16;
    const dim3 copy_grid(plan->P, (unsigned)std::max<int64_t>(1, std::min<int64_t>(cdiv(vec_per_patch, 1024), 64)));

    ActiveList act{nullptr, nullptr};
    if (reuse_mask) {
        ProfScope ps("mask_compact", st);
        compact_mask_kernel<<<1, 1024, 0, st>>>(reuse_mask, plan->P, cache->active, cache->count);
        PS_TRY(check_launch("compact_mask_kernel"));
        act.active = cache->active;
        act.count = cache->count;
    }
    if (cache->act_off && (reuse_mask || !cache->tiles_unmasked)) {
        // without a mask the query tiling depends on the plan only: built once and kept
        ProfScope ps("attn_tiles", st);
        PS_TRY(attention_tiles(request_offset, reuse_mask, plan->n, plan->S, cache->att_qt, cache->act_off, cache->tile_off, st));
        cache->tiles_unmasked = reuse_mask == nullptr;
    }
    const ActiveList all{nullptr, nullptr};
    const float qscale = 1.4426950408889634f / sqrtf((float)(d.heads > 0 ? C / d.heads : 1));

    auto gn_args = [&](const void* in, const void* gamma, const void* beta) {
        GroupNormArgs a;
        a.x = in; a.gamma = gamma; a.beta = beta; a.C = C; a.G = d.G; a.n = plan->n; a.eps = d.eps;
        a.nsplit = cache->nsplit; a.partial = cache->partial; a.scale_shift = cache->scale_shift;
        a.request_offset = request_offset; a.owner = owner; a.neighbour = plan->d_tab[PSERVE_TAB_NEIGHBOUR];
        return a;
    };
    auto base_gemm = [&](const void* A, int64_t lda, int K, int N, const void* B, const float* bias) {
        GemmArgs g{};
        g.A = A; g.lda = lda; g.conv = 0; g.geom = gm; g.act = act; g.tokens_are_rows = 1; g.M = (int32_t)T;
        g.N = N; g.K = K; g.taps = 1; g.B = B; g.bias = bias; g.res = nullptr; g.ldr = 0;
        g.epi = EPI_ROUTE; g.seg_cols = N;
        for (auto& s : g.seg) { s.ptr = nullptr; s.ld = 0; s.transposed = 0; s.scale = 1.f; }
        return g;
    };
    // GroupNorm(+SiLU) of `in` into the padded buffer, halo ring, 3x3 convolution (+bias, +residual) into `out`
    // stats_next: the output feeds another norm, so the convolution may leave that norm's partial sums behind
    bool have_partials = false;                     // cache->partial was filled by the previous convolution
    auto norm_conv = [&](const void* in, const StageWeights& w, int ci, const void* res, void* out, bool stats_next,
                         const float* rowbias = nullptr, hipEvent_t rowbias_ready = nullptr) -> int {
        GroupNormArgs ga = gn_args(in, w.gn_g[ci], w.gn_b[ci]);
        if (have_partials) { ProfScope ps("gn_finalize", st); PS_TRY(gn_finalize(ga, gm, dt, plan->S / 64, st)); }
        else if (in_stats && in == x) {             // the block input: its moments came with the split
            GroupNormArgs gi = ga;
            gi.partial = cache->in_partial;
            ProfScope ps("gn_finalize", st);
            PS_TRY(gn_finalize(gi, gm, dt, cache->in_nch, st, /*per_channel=*/true));
        }
        else { ProfScope ps("gn_stats", st); PS_TRY(gn_stats(ga, gm, dt, st)); }
        have_partials = false;
        // reused patches are not convolved: of them only the border tokens are normalised (the neighbours' rings)
        ga.rim_only = reuse_mask;
        if (push) {             // normalise + stitch in one pass (push); otherwise the rims are gathered afterwards (pull)
            ProfScope ps("gn_apply_stitch", st);
            PS_TRY(gn_apply(ga, gm, dt, /*silu=*/true, /*padded=*/true, /*stitch=*/true, cache->apad, all, st));
        } else {
            { ProfScope ps("gn_apply", st); PS_TRY(gn_apply(ga, gm, dt, true, true, false, cache->apad, all, st)); }
            { ProfScope ps("halo_gather", st);
              PS_TRY(halo_gather(cache->apad, plan->d_tab[PSERVE_TAB_HALO_SRC], gm, C, plan->ring, dt, act, st)); }
        }
        GemmArgs g = base_gemm(cache->apad, C, C, C, w.w[ci], w.b[ci]);
        g.conv = 1; g.taps = 9; g.res = res; g.ldr = C;
        g.rowbias = rowbias; g.row_owner = owner;
        g.seg[0].ptr = out; g.seg[0].ld = C;
        if (stats_next && !reuse_mask) {
            // (with a mask the reused patches keep cached activations this convolution never sees: gn_stats reads them)
            g.stats = cache->partial; g.stats_G = d.G; g.stats_slots = plan->S / 64;
            if (gemm_emits_stats(g, dt, mode)) have_partials = true;
            else { g.stats = nullptr; g.stats_G = 0; g.stats_slots = 0; }
        }
        if (rowbias_ready) PS_CHECK_HIP(hipStreamWaitEvent(st, rowbias_ready, 0));   // produced on the side stream
        ProfScope ps("conv3x3", st);
        return gemm(g, dt, mode, st);
    };

    // text keys / values of every request (cross-attention): input ctx only
    auto ctx_kv = [&](const StageWeights& w, hipStream_t s2) -> int {
        GemmArgs gk = base_gemm(ctx, d.ctx_dim, d.ctx_dim, 2 * C, w.w[2], nullptr);
        gk.tokens_are_rows = 0; gk.act = all; gk.M = plan->n * d.ctx_len; gk.seg_cols = C;
        gk.row_group = d.ctx_len; gk.row_group_pad = cache->cross_ld;
        const int64_t ctx_rows = (int64_t)plan->n * cache->cross_ld;
        gk.seg[0].ptr = cache->kc; gk.seg[0].ld = C;
        gk.seg[1].ptr = cache->vc; gk.seg[1].ld = cache->v_transposed ? ctx_rows : C; gk.seg[1].transposed = cache->v_transposed;
        ProfScope ps("linear_ctx_kv", s2);
        return gemm(gk, dt, mode, s2);
    };
    // SiLU -> linear on the per-request vector of stage si: cache->temb_e[si] [n][width] in slot order
    auto temb_proj = [&](const StageWeights& w, int si, int width, hipStream_t s2, float* dst = nullptr) -> int {
        if (!dst) dst = cache->temb_e[si];
        ProfScope ps("temb_proj", s2);
        const int32_t* perm = plan->d_tab[PSERVE_TAB_PERM];
        if (plan->n >= 2 && width >= 2048 && width % 2 == 0) {      // wide: pairs of slots
            const int64_t pairs = cdiv(plan->n, 2);
            const int cpb = pairs * cdiv(width, 64) <= 256 ? 64 : 128;    // channels per block: at most ~one block per CU
            const dim3 wgrid((unsigned)pairs, (unsigned)cdiv(width, cpb));
            const size_t wlds = sizeof(float) * (2 * d.temb_dim + 2 * 1024 * 2);     // SiLU(temb) x 2, partial sums
            if (wlds <= 64 * 1024) {
#define PS_TW(TT, LPR_) temb_proj_wide_kernel<TT, LPR_><<<wgrid, 1024, wlds, s2>>>((const TT*)temb, (const TT*)w.wt, w.bt, perm, \
                                                                                 plan->n, d.temb_dim, width, dst)
                if (dt == PSERVE_BF16) { if (cpb == 64) PS_TW(uint16_t, 32); else PS_TW(uint16_t, 64); }
                else { if (cpb == 64) PS_TW(float, 32); else PS_TW(float, 64); }
#undef PS_TW
                return check_launch("temb_proj_wide_kernel");
            }
        }
        const dim3 grid(plan->n, (unsigned)cdiv(width, 64));
        const size_t lds = sizeof(float) * (d.temb_dim + TEMB_KG * 64);
        if (dt == PSERVE_BF16)
            temb_proj_kernel<uint16_t><<<grid, 1024, lds, s2>>>((const uint16_t*)temb, (const uint16_t*)w.wt, w.bt, perm,
                                                               d.temb_dim, width, dst);
        else
            temb_proj_kernel<float><<<grid, 1024, lds, s2>>>((const float*)temb, (const float*)w.wt, w.bt, perm,
                                                            d.temb_dim, width, dst);
        return check_launch("temb_proj_kernel");
    };
    // all projections of stage k (one for RES2T and the adaLN sub-layers, one per stream for a joint block)
    auto temb_stage = [&](int k, hipStream_t s2) -> int {
        if (d.stages[k] == PSERVE_MMDIT) {
            PS_TRY(temb_proj(block->sw[k], k, 6 * C, s2, cache->temb_e[k]));
            return temb_proj(block->sw_txt[k], k, 6 * C, s2, cache->temb_e2[k]);
        }
        return temb_proj(block->sw[k], k, d.stages[k] == PSERVE_RES2T ? C : 3 * C, s2);
    };
    if (cache->side) {                              // fork: the side stream starts where this call starts
        PS_CHECK_HIP(hipEventRecord(cache->ev_fork, st));
        PS_CHECK_HIP(hipStreamWaitEvent(cache->side, cache->ev_fork, 0));
        for (int k = 0; k < d.n_stages; ++k)        // the short projections first: their consumers come early
            if (cache->side_temb && needs_temb(d.stages[k])) {
                PS_TRY(temb_stage(k, cache->side));
                PS_CHECK_HIP(hipEventRecord(cache->ev_temb[k], cache->side));
            }
        if (cache->side_stage >= 0) {
            PS_TRY(ctx_kv(block->sw[cache->side_stage], cache->side));
            PS_CHECK_HIP(hipEventRecord(cache->ev_join, cache->side));
        }
    }

    // attention of the queries in cache->q over the keys / values of stage si (self; `joint`: key count from SEQ_LEN,
    // all patches are queries) or over the text keys / values (cross), into cache->o
    auto run_attention = [&](int si, bool cross, bool joint) -> int {
        AttnArgs aa{};
        aa.Q = cache->q; aa.O = cache->o; aa.C = C; aa.heads = d.heads; aa.d = C / d.heads; aa.geom = gm;
        aa.K = cross ? cache->kc : cache->k[si];
        aa.V = cross ? cache->vc : cache->v[si];
        aa.v_transposed = cache->v_transposed;
        aa.ldv = !cache->v_transposed ? C : cross ? (int64_t)plan->n * cache->cross_ld : T;
        aa.act = joint ? all : act;
        aa.owner = owner; aa.perm = plan->d_tab[PSERVE_TAB_PERM];
        aa.cu_seqlens = plan->d_tab[PSERVE_TAB_CU_SEQLENS];
        aa.seq_len = joint ? plan->d_tab[PSERVE_TAB_SEQ_LEN] : nullptr;
        aa.cross_len = cross ? d.ctx_len : 0; aa.cross_ld = cross ? cache->cross_ld : 0;
        aa.act_off = cache->act_off; aa.tile_off = cache->tile_off; aa.n = plan->n; aa.max_tiles = cache->max_tiles;
        aa.qt = cache->att_qt; aa.max_rows = plan->max_tokens_per_image;
        ProfScope ps(cross ? "attn_cross" : "attn_self", st);
        return attention(aa, dt, mode, st);
    };
    // fused q / k / v projection of `in` (rows of the patches in `rows`) into cache->q (scaled), k[si], v[si]
    auto qkv_proj = [&](const void* in, const void* wqkv, int si, ActiveList rows, hipStream_t sq = nullptr) -> int {
        if (!sq) sq = st;
        GemmArgs g = base_gemm(in, C, C, 3 * C, wqkv, nullptr);
        g.act = rows; g.seg_cols = C;
        g.seg[0].ptr = cache->q; g.seg[0].ld = C; g.seg[0].scale = qscale;
        g.seg[1].ptr = cache->k[si]; g.seg[1].ld = C;
        g.seg[2].ptr = cache->v[si]; g.seg[2].ld = cache->v_transposed ? T : C; g.seg[2].transposed = cache->v_transposed;
        ProfScope ps("linear_qkv", sq);
        return gemm(g, dt, mode, sq);
    };
    // the projection of stage si as seen from the main stream: wait for the side stream, or run it here
    auto temb_ready = [&](const StageWeights&, int si, int) -> int {
        if (cache->side_temb) { PS_CHECK_HIP(hipStreamWaitEvent(st, cache->ev_temb[si], 0)); return PSERVE_OK; }
        return temb_stage(si, st);
    };

    const void* cur = x;
    for (int si = 0; si < d.n_stages; ++si) {
        const StageWeights& w = block->sw[si];
        const bool last = si == d.n_stages - 1;
        void* out;
        if (last) out = y;
        else if (cache->with_slots && d.stages[si + 1] == PSERVE_SATTN) out = cache->r[si + 1];   // producer writes the slot
        else out = (cur == cache->ping[0]) ? cache->ping[1] : cache->ping[0];

        switch (d.stages[si]) {
        case PSERVE_RES1:
            PS_TRY(norm_conv(cur, w, 0, cur, out, false));
            break;
        case PSERVE_RES2:
            PS_TRY(norm_conv(cur, w, 0, nullptr, cache->h1[si], true));
            PS_TRY(norm_conv(cache->h1[si], w, 1, cur, out, false));
            break;
        case PSERVE_RES2T: {
            // the projected embedding comes from the side stream; the first convolution adds it in its epilogue
            if (!cache->side_temb) PS_TRY(temb_stage(si, st));
            PS_TRY(norm_conv(cur, w, 0, nullptr, cache->h1[si], true, cache->temb_e[si], cache->side_temb ? cache->ev_temb[si] : nullptr));
            PS_TRY(norm_conv(cache->h1[si], w, 1, cur, out, false));
            break;
        }
        case PSERVE_SATTN:
        case PSERVE_LSATTN:
        case PSERVE_ASATTN: {
            const bool ada = d.stages[si] == PSERVE_ASATTN;
            const bool ln = d.stages[si] == PSERVE_LSATTN || ada;
            if (ada) PS_TRY(temb_ready(w, si, 3 * C));          // [shift | scale | gate] per request
            const void* rin = cur;
            if (!ln && cache->with_slots && cur != cache->r[si]) {    // first stage: merge fresh input into the slot
                ProfScope ps("reuse_copy", st);
                copy_patches_kernel<<<copy_grid, 256, 0, st>>>((const uint4*)cur, (uint4*)cache->r[si], vec_per_patch,
                                                               reuse_mask, reuse_mask ? 1 : 0);
                PS_TRY(check_launch("copy_patches_kernel"));
                rin = cache->r[si];
            }
            if (ln) {                                                 // per token: nothing of the reused patches is needed
                ProfScope ps("layer_norm", st);
                PS_TRY(layer_norm(rin, ada ? nullptr : w.gn_g[0], ada ? nullptr : w.gn_b[0], ada ? cache->temb_e[si] : nullptr,
                                  3 * C, owner, C, d.eps, gm, dt, cache->u, act, st));
            } else {
                GroupNormArgs ga = gn_args(rin, w.gn_g[0], w.gn_b[0]);
                if (in_stats && rin == x) {         // the block input itself (not the slot that mixes in cached patches)
                    GroupNormArgs gi = ga;
                    gi.partial = cache->in_partial;
                    ProfScope ps("gn_finalize", st);
                    PS_TRY(gn_finalize(gi, gm, dt, cache->in_nch, st, /*per_channel=*/true));
                } else { ProfScope ps("gn_stats", st); PS_TRY(gn_stats(ga, gm, dt, st)); }
                { ProfScope ps("gn_apply", st); PS_TRY(gn_apply(ga, gm, dt, false, false, false, cache->u, act, st)); }
            }
            PS_TRY(qkv_proj(cache->u, w.w[0], si, act));
            PS_TRY(run_attention(si, /*cross=*/false, /*joint=*/false));
            GemmArgs go = base_gemm(cache->o, C, C, C, w.w[1], w.b[1]);
            go.res = rin; go.ldr = C;
            if (ada) { go.rowscale = cache->temb_e[si] + 2 * C; go.rowscale_ld = 3 * C; go.row_owner = owner; }
            go.seg[0].ptr = out; go.seg[0].ld = C;
            { ProfScope ps("linear_out", st); PS_TRY(gemm(go, dt, mode, st)); }
            break;
        }
        case PSERVE_MMDIT: {
            // Two streams (image patches, text patches) with their own weights, as two patch lists over the joint
            // token matrix; one attention per request over all its tokens.
            const int F = d.ffn_mult * C;
            PS_TRY(temb_ready(w, si, 6 * C));
            void* mid = (cur == cache->ping[0] || out == cache->ping[0]) ? ((cur == cache->ping[1] || out == cache->ping[1]) ? cache->q : cache->ping[1]) : cache->ping[0];
            // The text stream's kernels go to the side stream: they touch the rows of the text patches only (every
            // buffer is shared row-wise), so the two streams meet at the attention and at the end of the stage.
            hipStream_t sx[2] = {st, cache->side ? cache->side : st};
            auto fork_txt = [&](int e) -> int {           // the side stream continues from this point of the main one
                if (sx[1] == st) return PSERVE_OK;
                PS_CHECK_HIP(hipEventRecord(cache->ev_txt[e], st));
                PS_CHECK_HIP(hipStreamWaitEvent(sx[1], cache->ev_txt[e], 0));
                return PSERVE_OK;
            };
            auto join_txt = [&](int e) -> int {           // the main stream waits for what the side stream has queued
                if (sx[1] == st) return PSERVE_OK;
                PS_CHECK_HIP(hipEventRecord(cache->ev_txt[e], sx[1]));
                PS_CHECK_HIP(hipStreamWaitEvent(st, cache->ev_txt[e], 0));
                return PSERVE_OK;
            };
            PS_TRY(fork_txt(0));
            for (int xs = 0; xs < 2; ++xs) {
                const StageWeights& v = xs == 0 ? block->sw[si] : block->sw_txt[si];
                const float* mod = xs == 0 ? cache->temb_e[si] : cache->temb_e2[si];
                const ActiveList ax{cache->stream_list[xs], cache->stream_count + xs};
                { ProfScope ps("layer_norm", sx[xs]);
                  PS_TRY(layer_norm(cur, nullptr, nullptr, mod, 6 * C, owner, C, d.eps, gm, dt, cache->u, ax, sx[xs])); }
                PS_TRY(qkv_proj(cache->u, v.w[0], si, ax, sx[xs]));
            }
            PS_TRY(join_txt(1));
            PS_TRY(run_attention(si, /*cross=*/false, /*joint=*/true));
            PS_TRY(fork_txt(2));
            for (int xs = 0; xs < 2; ++xs) {
                const StageWeights& v = xs == 0 ? block->sw[si] : block->sw_txt[si];
                const float* mod = xs == 0 ? cache->temb_e[si] : cache->temb_e2[si];
                const ActiveList ax{cache->stream_list[xs], cache->stream_count + xs};
                hipStream_t s_ = sx[xs];
                GemmArgs go = base_gemm(cache->o, C, C, C, v.w[1], v.b[1]);
                go.act = ax; go.res = cur; go.ldr = C;
                go.rowscale = mod + 2 * C; go.rowscale_ld = 6 * C; go.row_owner = owner;
                go.seg[0].ptr = mid; go.seg[0].ld = C;
                { ProfScope ps("linear_out", s_); PS_TRY(gemm(go, dt, mode, s_)); }
                { ProfScope ps("layer_norm", s_);
                  PS_TRY(layer_norm(mid, nullptr, nullptr, mod + 3 * C, 6 * C, owner, C, d.eps, gm, dt, cache->u, ax, s_)); }
                GemmArgs g1 = base_gemm(cache->u, C, C, F, v.w[3], v.b[3]);
                g1.act = ax; g1.act_gelu = 1;
                g1.seg[0].ptr = cache->hidden; g1.seg[0].ld = F;
                { ProfScope ps("mlp_in", s_); PS_TRY(gemm(g1, dt, mode, s_)); }
                GemmArgs g2 = base_gemm(cache->hidden, F, F, C, v.w[4], v.b[4]);
                g2.act = ax; g2.res = mid; g2.ldr = C;
                g2.rowscale = mod + 5 * C; g2.rowscale_ld = 6 * C; g2.row_owner = owner;
                g2.seg[0].ptr = out; g2.seg[0].ld = C;
                { ProfScope ps("mlp_out", s_); PS_TRY(gemm(g2, dt, mode, s_)); }
            }
            PS_TRY(join_txt(3));
            break;
        }
        case PSERVE_AMLP: {
            const int F = d.ffn_mult * C;
            PS_TRY(temb_ready(w, si, 3 * C));
            { ProfScope ps("layer_norm", st);
              PS_TRY(layer_norm(cur, nullptr, nullptr, cache->temb_e[si], 3 * C, owner, C, d.eps, gm, dt, cache->u, act, st)); }
            GemmArgs g1 = base_gemm(cache->u, C, C, F, w.w[0], w.b[0]);
            g1.act_gelu = 1;
            g1.seg[0].ptr = cache->hidden; g1.seg[0].ld = F;
            { ProfScope ps("mlp_in", st); PS_TRY(gemm(g1, dt, mode, st)); }
            GemmArgs g2 = base_gemm(cache->hidden, F, F, C, w.w[1], w.b[1]);
            g2.res = cur; g2.ldr = C;
            g2.rowscale = cache->temb_e[si] + 2 * C; g2.rowscale_ld = 3 * C; g2.row_owner = owner;
            g2.seg[0].ptr = out; g2.seg[0].ld = C;
            { ProfScope ps("mlp_out", st); PS_TRY(gemm(g2, dt, mode, st)); }
            break;
        }
        case PSERVE_XATTN:
        case PSERVE_LXATTN: {
            if (cache->side_stage == si) PS_CHECK_HIP(hipStreamWaitEvent(st, cache->ev_join, 0));     // join
            else PS_TRY(ctx_kv(w, st));
            const void* qin = cur;
            if (d.stages[si] == PSERVE_LXATTN) {
                ProfScope ps("layer_norm", st);
                PS_TRY(layer_norm(cur, w.gn_g[0], w.gn_b[0], nullptr, 0, nullptr, C, d.eps, gm, dt, cache->u, act, st));
                qin = cache->u;
            }
            GemmArgs gq = base_gemm(qin, C, C, C, w.w[0], nullptr);
            gq.seg[0].ptr = cache->q; gq.seg[0].ld = C; gq.seg[0].scale = qscale;
            { ProfScope ps("linear_q", st); PS_TRY(gemm(gq, dt, mode, st)); }
            PS_TRY(run_attention(si, /*cross=*/true, /*joint=*/false));
            GemmArgs go = base_gemm(cache->o, C, C, C, w.w[1], w.b[1]);
            go.res = cur; go.ldr = C;
            go.seg[0].ptr = out; go.seg[0].ld = C;
            { ProfScope ps("linear_out", st); PS_TRY(gemm(go, dt, mode, st)); }
            break;
        }
        case PSERVE_FFN:
        case PSERVE_LFFN: {
            const int F = d.ffn_mult * C;
            const void* fin = cur;
            if (d.stages[si] == PSERVE_LFFN) {
                ProfScope ps("layer_norm", st);
                PS_TRY(layer_norm(cur, w.gn_g[0], w.gn_b[0], nullptr, 0, nullptr, C, d.eps, gm, dt, cache->u, act, st));
                fin = cache->u;
            }
            GemmArgs g1 = base_gemm(fin, C, C, 2 * F, w.w[0], w.b[0]);
            g1.epi = EPI_GEGLU;
            g1.seg[0].ptr = cache->hidden; g1.seg[0].ld = F;
            { ProfScope ps("ffn_geglu", st); PS_TRY(gemm(g1, dt, mode, st)); }
            GemmArgs g2 = base_gemm(cache->hidden, F, F, C, w.w[1], w.b[1]);
            g2.res = cur; g2.ldr = C;
            g2.seg[0].ptr = out; g2.seg[0].ld = C;
            { ProfScope ps("ffn_out", st); PS_TRY(gemm(g2, dt, mode, st)); }
            break;
        }
        }
        cur = out;
    }
    if (cache->with_slots) {
        // computed patches refresh the output slot; reused patches take the cached output
        ProfScope ps("reuse_copy", st);
        copy_patches_kernel<<<copy_grid, 256, 0, st>>>((const uint4*)y, (uint4*)cache->yslot, vec_per_patch, reuse_mask,
                                                       reuse_mask ? 1 : 0);
        PS_TRY(check_launch("copy_patches_kernel"));
        if (reuse_mask) {
            copy_patches_kernel<<<copy_grid, 256, 0, st>>>((const uint4*)cache->yslot, (uint4*)y, vec_per_patch, reuse_mask, 2);
            PS_TRY(check_launch("copy_patches_kernel"));
        }
    }
    cache->filled = true;
    return PSERVE_OK;
}

}  // extern "C"
