// Patch planner (Compressed Sparse Patch tables + neighbour / halo metadata) and the
// split / reassembly copies between per-image NCHW latents and the patch-major token matrix.
//
// Paper: section "Compressed Sparse Patch Format" (requests reordered by resolution,
// RequestOffset, per-patch request index, resolution offsets) and section
// "Patch-Tailored Diffusion Operators" (neighbours recorded at split time, absent
// neighbour = zero fill).
#include "common.h"

#include <algorithm>
#include <numeric>
#include <string.h>

namespace pserve {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

// ---- kernels ----------------------------------------------------------------------------

// One block: exclusive scan of patch counts over sorted slots, resolution runs, token offsets.
// n is small (a serving batch), so a single wavefront-serial pass by thread 0 per 256-slot
// chunk would do; a block-wide Hillis-Steele scan keeps it O(log n) deep anyway.
__global__ void plan_offsets_kernel(const int32_t* __restrict__ sorted_hw, int32_t n, int32_t ph, int32_t pw,
                                    int32_t tp, int32_t text_len, int32_t* __restrict__ request_offset,
                                    int32_t* __restrict__ cu_seqlens, int32_t* __restrict__ res_offset,
                                    int32_t* __restrict__ res_hw, int32_t* __restrict__ seq_len) {
    __shared__ int32_t s_cnt[1024];
    __shared__ int32_t s_flag[1024];
    __shared__ int32_t carry_cnt, carry_flag;
    const int tid = threadIdx.x;
    if (tid == 0) { carry_cnt = 0; carry_flag = 0; request_offset[0] = 0; cu_seqlens[0] = 0; }
    __syncthreads();
    for (int base = 0; base < n; base += blockDim.x) {
        const int s = base + tid;
        int32_t cnt = 0, flag = 0;
        if (s < n) {
            const int32_t H = sorted_hw[2 * s], W = sorted_hw[2 * s + 1];
            cnt = (H / ph) * (W / pw) + tp;               // tp text patches ride behind the image patches
            seq_len[s] = H * W + text_len;                // valid tokens of the slot (padding of the last text patch excluded)
            flag = (s == 0) || sorted_hw[2 * s - 2] != H || sorted_hw[2 * s - 1] != W;   // first slot of a resolution run
        }
        s_cnt[tid] = cnt;
        s_flag[tid] = flag;
        __syncthreads();
        for (int off = 1; off < (int)blockDim.x; off <<= 1) {      // inclusive scan
            int32_t a = 0, b = 0;
            if (tid >= off) { a = s_cnt[tid - off]; b = s_flag[tid - off]; }
            __syncthreads();
            s_cnt[tid] += a;
            s_flag[tid] += b;
            __syncthreads();
        }
        if (s < n) {
            const int32_t incl = carry_cnt + s_cnt[tid];
            request_offset[s + 1] = incl;
            cu_seqlens[s + 1] = incl * ph * pw;
            if (flag) {
                const int32_t k = carry_flag + s_flag[tid] - 1;
                res_offset[k] = s;
                res_hw[2 * k] = sorted_hw[2 * s];
                res_hw[2 * k + 1] = sorted_hw[2 * s + 1];
            }
        }
        __syncthreads();
        if (tid == blockDim.x - 1) { carry_cnt += s_cnt[tid]; carry_flag += s_flag[tid]; }
        __syncthreads();
    }
    if (tid == 0) res_offset[carry_flag] = n;
}

// One thread per patch: owner by binary search in RequestOffset, grid position, 8 neighbours.
__global__ void plan_patches_kernel(const int32_t* __restrict__ sorted_hw, const int32_t* __restrict__ request_offset,
                                    int32_t n, int32_t P, int32_t ph, int32_t pw, int32_t* __restrict__ owner,
                                    int32_t* __restrict__ rc, int32_t* __restrict__ neighbour) {
    // (text patches: local index >= gh*gw; grid position (-1, k), no neighbours)
    const int p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= P) return;
    int lo = 0, hi = n;                       // largest s with request_offset[s] <= p
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (request_offset[mid] <= p) lo = mid; else hi = mid;
    }
    const int s = lo;
    const int gh = sorted_hw[2 * s] / ph, gw = sorted_hw[2 * s + 1] / pw;
    const int local = p - request_offset[s];
    owner[p] = s;
    if (local >= gh * gw) {
        rc[2 * p] = -1;
        rc[2 * p + 1] = local - gh * gw;
        for (int k = 0; k < 8; ++k) neighbour[8 * p + k] = -1;
        return;
    }
    const int r = local / gw, c = local - r * gw;
    rc[2 * p] = r;
    rc[2 * p + 1] = c;
    int k = 0;
    for (int dy = -1; dy <= 1; ++dy)
        for (int dx = -1; dx <= 1; ++dx) {
            if (dy == 0 && dx == 0) continue;
            const int rr = r + dy, cc = c + dx;
            neighbour[8 * p + k] = (rr >= 0 && rr < gh && cc >= 0 && cc < gw) ? request_offset[s] + rr * gw + cc : -1;
            ++k;
        }
}

// One thread per (patch, ring entry): global token id of the pixel one step outside the patch.
__global__ void plan_halo_kernel(const int32_t* __restrict__ sorted_hw, const int32_t* __restrict__ request_offset,
                                 const int32_t* __restrict__ owner, const int32_t* __restrict__ rc, int32_t P,
                                 int32_t ph, int32_t pw, int32_t ring, int32_t* __restrict__ halo_src) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)P * ring) return;
    const int p = (int)(i / ring), k = (int)(i - (int64_t)p * ring);
    int y, x;                                 // ring pixel relative to the patch origin
    if (k < pw + 2) { y = -1; x = k - 1; }
    else if (k < 2 * (pw + 2)) { y = ph; x = k - (pw + 2) - 1; }
    else if (k < 2 * (pw + 2) + ph) { y = k - 2 * (pw + 2); x = -1; }
    else { y = k - 2 * (pw + 2) - ph; x = pw; }
    const int s = owner[p];
    const int H = sorted_hw[2 * s], W = sorted_hw[2 * s + 1], gw = W / pw;
    const int Y = rc[2 * p] * ph + y, X = rc[2 * p + 1] * pw + x;      // absolute pixel in the image
    int32_t tok = -1;
    if (rc[2 * p] >= 0 && Y >= 0 && Y < H && X >= 0 && X < W) {
        const int q = request_offset[s] + (Y / ph) * gw + (X / pw);
        tok = q * ph * pw + (Y % ph) * pw + (X % pw);
    }
    halo_src[i] = tok;
}

// ---- split / reassemble -------------------------------------------------------------------
constexpr int IMG_CHUNK = 32;
struct ImagePtrs {
    void* p[IMG_CHUNK];       // image of sorted slot slot0 + k
};

// Block = one patch row (patch p, row y) x 64 channels; 32-pixel chunks are transposed through LDS.
// TO_PATCH: NCHW image -> x[T][C]; else the reverse.
template <typename T, bool TO_PATCH>
__global__ void __launch_bounds__(256)
split_kernel(ImagePtrs imgs, int slot0, int patch0, const int32_t* __restrict__ sorted_hw,
             const int32_t* __restrict__ owner, const int32_t* __restrict__ rc, int32_t ph, int32_t pw, int32_t C,
             T* __restrict__ x) {
    __shared__ T tile[64][33];
    const int p = patch0 + blockIdx.x / ph;
    const int y = blockIdx.x % ph;
    const int c0 = blockIdx.y * 64;
    if (rc[2 * p] < 0) return;                  // a text patch: not part of any image
    const int s = owner[p];
    const int H = sorted_hw[2 * s], W = sorted_hw[2 * s + 1];
    T* img = (T*)imgs.p[s - slot0];
    const int Y = rc[2 * p] * ph + y, X0 = rc[2 * p + 1] * pw;
    const int64_t tok0 = (int64_t)p * ph * pw + (int64_t)y * pw;
    const int tid = threadIdx.x;
    for (int xc = 0; xc < pw; xc += 32) {
        if (TO_PATCH) {
            for (int i = tid; i < 64 * 32; i += 256) {
                const int px = i & 31, ch = i >> 5;
                if (xc + px < pw && c0 + ch < C)
                    tile[ch][px] = img[((int64_t)(c0 + ch) * H + Y) * W + X0 + xc + px];
            }
            __syncthreads();
            for (int i = tid; i < 64 * 32; i += 256) {
                const int ch = i & 63, px = i >> 6;
                if (xc + px < pw && c0 + ch < C) x[(tok0 + xc + px) * C + c0 + ch] = tile[ch][px];
            }
        } else {
            for (int i = tid; i < 64 * 32; i += 256) {
                const int ch = i & 63, px = i >> 6;
                if (xc + px < pw && c0 + ch < C) tile[ch][px] = x[(tok0 + xc + px) * C + c0 + ch];
            }
            __syncthreads();
            for (int i = tid; i < 64 * 32; i += 256) {
                const int px = i & 31, ch = i >> 5;
                if (xc + px < pw && c0 + ch < C)
                    img[((int64_t)(c0 + ch) * H + Y) * W + X0 + xc + px] = tile[ch][px];
            }
        }
        __syncthreads();
    }
}

// bf16 fast path: tile = 64 channels x 32 consecutive tokens of one patch, one 16-byte access per thread on each
// side (8 pixels of one channel row in NCHW; 8 channels of one token in the patch-major layout), transposed in LDS.
// Needs pw % 8 == 0, (ph*pw) % 32 == 0, C % 64 == 0, W % 8 == 0 and 16-byte aligned images.
template <bool TO_PATCH>
__global__ void __launch_bounds__(256)
split_vec_kernel(ImagePtrs imgs, int slot0, int patch0, const int32_t* __restrict__ sorted_hw,
                 const int32_t* __restrict__ owner, const int32_t* __restrict__ rc, int32_t ph, int32_t pw, int32_t C,
                 uint16_t* __restrict__ x) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[32][72];      // [token][channel], rows padded to 144 bytes
    const int S = ph * pw, tiles = S / 32;
    const int p = patch0 + blockIdx.x / tiles;
    const int t0 = (blockIdx.x % tiles) * 32;
    const int c0 = blockIdx.y * 64;
    if (rc[2 * p] < 0) return;                  // a text patch: not part of any image
    const int s = owner[p];
    const int H = sorted_hw[2 * s], W = sorted_hw[2 * s + 1];
    uint16_t* img = (uint16_t*)imgs.p[s - slot0];
    const int tid = threadIdx.x;
    // image side: channel ich, 8 pixels starting at token t0 + 8*iq
    const int ich = tid >> 2, iq = tid & 3;
    const int it = t0 + 8 * iq, iy = it / pw, ix = it - iy * pw;
    uint16_t* ip = img + ((int64_t)(c0 + ich) * H + rc[2 * p] * ph + iy) * W + rc[2 * p + 1] * pw + ix;
    // patch side: token t0 + ptk, channels 8*pq .. +8
    const int ptk = tid >> 3, pq = tid & 7;
    uint16_t* xp = x + ((int64_t)p * S + t0 + ptk) * C + c0 + 8 * pq;
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    if (TO_PATCH) {
        const u32x4 v = *reinterpret_cast<const u32x4*>(ip);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            tile[8 * iq + 2 * k][ich] = (uint16_t)(v[k] & 0xFFFFu);
            tile[8 * iq + 2 * k + 1][ich] = (uint16_t)(v[k] >> 16);
        }
        __syncthreads();
        *reinterpret_cast<u32x4*>(xp) = *reinterpret_cast<const u32x4*>(&tile[ptk][8 * pq]);
    } else {
        *reinterpret_cast<u32x4*>(&tile[ptk][8 * pq]) = *reinterpret_cast<const u32x4*>(xp);
        __syncthreads();
        u32x4 v;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            v[k] = (uint32_t)tile[8 * iq + 2 * k][ich] | ((uint32_t)tile[8 * iq + 2 * k + 1][ich] << 16);
        *reinterpret_cast<u32x4*>(ip) = v;
    }
}

// Split (bf16 fast path) that also leaves the moments of every channel behind, for a GroupNorm that reads x next:
// block = (patch, one of `nch` token chunks, 64 channels); it walks the chunk's 32-token tiles like split_vec_kernel
// and keeps, per thread, the sums of (x - K) and (x - K)^2 of its eight channels (K = the channel's value in the
// chunk's first token: nothing is lost when the mean is far from zero).  Per (patch, chunk, channel) it stores the
// mean and the sum of squared deviations M2 of the chunk's tokens: stats[((p * nch + chunk) * C + c) * 2 + {0, 1}],
// which the GroupNorm finalize merges (fixed order, no atomics).
__global__ void __launch_bounds__(256)
split_stats_kernel(ImagePtrs imgs, int slot0, int patch0, const int32_t* __restrict__ sorted_hw,
                   const int32_t* __restrict__ owner, const int32_t* __restrict__ rc, int32_t ph, int32_t pw, int32_t C,
                   int32_t nch, uint16_t* __restrict__ x, float* __restrict__ stats) {
    __shared__ __attribute__((aligned(16))) uint16_t tile[32][72];      // [token][channel], rows padded to 144 bytes
    __shared__ float red[2][32][65];
    __shared__ float kk[64];
    const int S = ph * pw, tiles = S / 32, tpc = tiles / nch;
    const int p = patch0 + blockIdx.x / nch, tc = blockIdx.x % nch;
    const int c0 = blockIdx.y * 64;
    if (rc[2 * p] < 0) return;                  // a text patch: not part of any image
    const int s = owner[p];
    const int H = sorted_hw[2 * s], W = sorted_hw[2 * s + 1];
    const uint16_t* img = (const uint16_t*)imgs.p[s - slot0];
    const int tid = threadIdx.x;
    const int ich = tid >> 2, iq = tid & 3;     // image side: channel ich, 8 pixels starting at token t0 + 8*iq
    const int ptk = tid >> 3, pq = tid & 7;     // patch side: token t0 + ptk, channels 8*pq .. +8
    const uint16_t* ibase = img + ((int64_t)(c0 + ich) * H + rc[2 * p] * ph) * W + rc[2 * p + 1] * pw;
    typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
    float s1[8], s2[8], k0[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { s1[e] = 0.f; s2[e] = 0.f; k0[e] = 0.f; }
    for (int ti = 0; ti < tpc; ++ti) {
        const int t0 = (tc * tpc + ti) * 32;
        const int it = t0 + 8 * iq, iy = it / pw, ix = it - iy * pw;
        const u32x4 v = *reinterpret_cast<const u32x4*>(ibase + (int64_t)iy * W + ix);
        if (ti) __syncthreads();                // the previous tile has been read
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            tile[8 * iq + 2 * k][ich] = (uint16_t)(v[k] & 0xFFFFu);
            tile[8 * iq + 2 * k + 1][ich] = (uint16_t)(v[k] >> 16);
        }
        __syncthreads();
        const u32x4 o = *reinterpret_cast<const u32x4*>(&tile[ptk][8 * pq]);
        if (ti == 0) {
            const u32x4 f = *reinterpret_cast<const u32x4*>(&tile[0][8 * pq]);
#pragma unroll
            for (int k = 0; k < 4; ++k) { k0[2 * k] = __uint_as_float(f[k] << 16); k0[2 * k + 1] = __uint_as_float(f[k] & 0xFFFF0000u); }
        }
        *reinterpret_cast<u32x4*>(x + ((int64_t)p * S + t0 + ptk) * C + c0 + 8 * pq) = o;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float lo = __uint_as_float(o[k] << 16) - k0[2 * k], hi = __uint_as_float(o[k] & 0xFFFF0000u) - k0[2 * k + 1];
            s1[2 * k] += lo; s2[2 * k] = fmaf(lo, lo, s2[2 * k]);
            s1[2 * k + 1] += hi; s2[2 * k + 1] = fmaf(hi, hi, s2[2 * k + 1]);
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) { red[0][ptk][8 * pq + e] = s1[e]; red[1][ptk][8 * pq + e] = s2[e]; }
    if (ptk == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) kk[8 * pq + e] = k0[e];
    }
    __syncthreads();
    if (tid < 64) {
        float a = 0.f, b = 0.f;
        for (int l = 0; l < 32; ++l) { a += red[0][l][tid]; b += red[1][l][tid]; }      // fixed order
        const float nt = (float)(tpc * 32), inv = 1.f / nt;
        float* dst = stats + (((int64_t)p * nch + tc) * C + c0 + tid) * 2;
        dst[0] = kk[tid] + a * inv;
        dst[1] = fmaxf(b - a * a * inv, 0.f);
    }
}

// Text tokens of every request <-> the text patches of the joint token matrix.  One thread per (slot, text row
// incl. padding, 16-byte vector).  TO_PATCH: text [n][L][C] (caller order) -> x, padding rows zeroed; else x -> text.
template <bool TO_PATCH>
__global__ void text_rows_kernel(uint4* __restrict__ x, uint4* __restrict__ text, const int32_t* __restrict__ perm,
                                 const int32_t* __restrict__ cu_seqlens, const int32_t* __restrict__ seq_len, int32_t n,
                                 int32_t L, int32_t rows_pad, int32_t CV) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)n * rows_pad * CV) return;
    const int cv = (int)(i % CV);
    const int r = (int)((i / CV) % rows_pad);
    const int s = (int)(i / ((int64_t)CV * rows_pad));
    const int64_t xrow = (int64_t)cu_seqlens[s] + seq_len[s] - L + r;         // first text row sits behind the image tokens
    if (TO_PATCH) x[xrow * CV + cv] = r < L ? text[((int64_t)perm[s] * L + r) * CV + cv] : make_uint4(0, 0, 0, 0);
    else if (r < L) text[((int64_t)perm[s] * L + r) * CV + cv] = x[xrow * CV + cv];
}

template <bool TO_PATCH>
static int run_text(const pserve_plan_t* plan, void* x, void* text, int32_t C, int dtype, hipStream_t st) {
    PS_REQUIRE(plan && x && text, "text scatter/gather: NULL argument");
    PS_REQUIRE(plan->text_len > 0, "text scatter/gather: the plan has no text patches (pserve_plan_text)");
    PS_REQUIRE(dtype == PSERVE_F32 || dtype == PSERVE_BF16, "text scatter/gather: unknown dtype %d", dtype);
    const int vn = dtype == PSERVE_BF16 ? 8 : 4;
    PS_REQUIRE(C > 0 && C % vn == 0, "text scatter/gather: C=%d must be a multiple of 16 bytes", C);
    const int rows_pad = plan->text_patches * plan->S, CV = C / vn;
    const int64_t items = (int64_t)plan->n * rows_pad * CV;
    text_rows_kernel<TO_PATCH><<<(unsigned)cdiv(items, 256), 256, 0, st>>>((uint4*)x, (uint4*)text, plan->d_tab[PSERVE_TAB_PERM],
        plan->d_tab[PSERVE_TAB_CU_SEQLENS], plan->d_tab[PSERVE_TAB_SEQ_LEN], plan->n, plan->text_len, rows_pad, CV);
    return check_launch("text_rows_kernel");
}

template <bool TO_PATCH>
static int run_split(const pserve_plan_t* plan, void* const* images, int32_t C, int dtype, void* x, hipStream_t st) {
    PS_REQUIRE(plan && images && x, "split/reassemble: NULL argument");
    PS_REQUIRE(C > 0, "split/reassemble: C must be positive");
    PS_REQUIRE(dtype == PSERVE_F32 || dtype == PSERVE_BF16, "split/reassemble: unknown dtype %d", dtype);
    const auto& ro = plan->h_tab[PSERVE_TAB_REQUEST_OFFSET];
    const auto& perm = plan->h_tab[PSERVE_TAB_PERM];
    for (int i = 0; i < plan->n; ++i) PS_REQUIRE(images[i], "split/reassemble: image %d is NULL", i);
    for (int s0 = 0; s0 < plan->n; s0 += IMG_CHUNK) {
        const int s1 = std::min(plan->n, s0 + IMG_CHUNK);
        ImagePtrs ip;
        memset(&ip, 0, sizeof(ip));
        for (int s = s0; s < s1; ++s) ip.p[s - s0] = images[perm[s]];
        const int patch0 = ro[s0], npatch = ro[s1] - ro[s0];
        bool vec = dtype == PSERVE_BF16 && plan->pw % 8 == 0 && plan->S % 32 == 0 && C % 64 == 0 && ((uintptr_t)x & 15) == 0;
        for (int s = s0; s < s1 && vec; ++s)
            vec = plan->h_sorted_hw[2 * s + 1] % 8 == 0 && ((uintptr_t)ip.p[s - s0] & 15) == 0;
        if (vec) {
            dim3 vgrid(npatch * (plan->S / 32), (unsigned)(C / 64));
            split_vec_kernel<TO_PATCH><<<vgrid, 256, 0, st>>>(ip, s0, patch0, plan->d_sorted_hw,
                plan->d_tab[PSERVE_TAB_PATCH_OWNER], plan->d_tab[PSERVE_TAB_PATCH_RC], plan->ph, plan->pw, C, (uint16_t*)x);
            PS_TRY(check_launch("split_vec_kernel"));
            continue;
        }
        dim3 grid(npatch * plan->ph, (unsigned)cdiv(C, 64));
        if (dtype == PSERVE_BF16)
            split_kernel<uint16_t, TO_PATCH><<<grid, 256, 0, st>>>(ip, s0, patch0, plan->d_sorted_hw,
                plan->d_tab[PSERVE_TAB_PATCH_OWNER], plan->d_tab[PSERVE_TAB_PATCH_RC], plan->ph, plan->pw, C, (uint16_t*)x);
        else
            split_kernel<float, TO_PATCH><<<grid, 256, 0, st>>>(ip, s0, patch0, plan->d_sorted_hw,
                plan->d_tab[PSERVE_TAB_PATCH_OWNER], plan->d_tab[PSERVE_TAB_PATCH_RC], plan->ph, plan->pw, C, (float*)x);
        PS_TRY(check_launch("split_kernel"));
    }
    return PSERVE_OK;
}


// pserve_split (bf16 fast path only) that also writes the per-channel moments of x; *done = false (and nothing is
// written) where the fast path does not apply
int split_with_stats(const pserve_plan_t* plan, const void* const* images, int32_t C, void* x, float* stats, int32_t nch,
                     hipStream_t st, bool* done) {
    *done = false;
    const auto& ro = plan->h_tab[PSERVE_TAB_REQUEST_OFFSET];
    const auto& perm = plan->h_tab[PSERVE_TAB_PERM];
    bool vec = plan->pw % 8 == 0 && plan->S % 32 == 0 && C % 64 == 0 && ((uintptr_t)x & 15) == 0 && nch >= 1 &&
               (plan->S / 32) % nch == 0 && plan->text_len == 0;
    for (int i = 0; i < plan->n && vec; ++i)
        vec = images[i] && plan->h_sorted_hw[2 * i + 1] % 8 == 0 && ((uintptr_t)images[i] & 15) == 0;
    if (!vec) return PSERVE_OK;
    for (int s0 = 0; s0 < plan->n; s0 += IMG_CHUNK) {
        const int s1 = std::min(plan->n, s0 + IMG_CHUNK);
        ImagePtrs ip;
        memset(&ip, 0, sizeof(ip));
        for (int s = s0; s < s1; ++s) ip.p[s - s0] = (void*)images[perm[s]];
        const int patch0 = ro[s0], npatch = ro[s1] - ro[s0];
        dim3 grid(npatch * nch, (unsigned)(C / 64));
        split_stats_kernel<<<grid, 256, 0, st>>>(ip, s0, patch0, plan->d_sorted_hw, plan->d_tab[PSERVE_TAB_PATCH_OWNER],
                                                 plan->d_tab[PSERVE_TAB_PATCH_RC], plan->ph, plan->pw, C, nch, (uint16_t*)x, stats);
        PS_TRY(check_launch("split_stats_kernel"));
    }
    *done = true;
    return PSERVE_OK;
}
}  // namespace pserve

using namespace pserve;

extern "C" {

const char* pserve_last_error(void) { return g_err; }

int pserve_plan(const int32_t* res, int32_t n, int32_t ph, int32_t pw, void* stream, pserve_plan_t** out) {
    return pserve_plan_text(res, n, ph, pw, 0, stream, out);
}

int pserve_text_scatter(const pserve_plan_t* plan, const void* text, int32_t C, int dtype, void* x, void* stream) {
    return run_text<true>(plan, x, const_cast<void*>(text), C, dtype, (hipStream_t)stream);
}

int pserve_text_gather(const pserve_plan_t* plan, const void* x, int32_t C, int dtype, void* text, void* stream) {
    return run_text<false>(plan, const_cast<void*>(x), text, C, dtype, (hipStream_t)stream);
}

static int plan_text_impl(const int32_t* res, int32_t n, int32_t ph, int32_t pw, int32_t text_len, void* stream,
                     pserve_plan_t** out) {
    PS_REQUIRE(out, "pserve_plan: out is NULL");
    PS_REQUIRE(text_len >= 0, "pserve_plan: negative text_len");
    *out = nullptr;
    PS_REQUIRE(res && n > 0, "pserve_plan: need n > 0 resolutions");
    PS_REQUIRE((ph == 0) == (pw == 0) && ph >= 0 && pw >= 0, "pserve_plan: patch must be (0,0) or both positive");
    for (int i = 0; i < n; ++i)
        PS_REQUIRE(res[2 * i] > 0 && res[2 * i + 1] > 0, "pserve_plan: request %d has a non-positive size", i);
    if (ph == 0) {                                            // patch-size rule: gcd per dimension
        for (int i = 0; i < n; ++i) { ph = std::gcd(ph, res[2 * i]); pw = std::gcd(pw, res[2 * i + 1]); }
    }
    int64_t P = 0, max_tok = 0;
    for (int i = 0; i < n; ++i) {
        PS_REQUIRE(res[2 * i] % ph == 0 && res[2 * i + 1] % pw == 0,
                   "pserve_plan: request %d (%dx%d) is not a multiple of the patch %dx%d", i, res[2 * i], res[2 * i + 1], ph, pw);
        P += (int64_t)(res[2 * i] / ph) * (res[2 * i + 1] / pw);
        max_tok = std::max<int64_t>(max_tok, (int64_t)res[2 * i] * res[2 * i + 1]);
    }
    const int32_t tp = (int32_t)cdiv(text_len, (int64_t)ph * pw);     // text patches per request
    P += (int64_t)n * tp;
    max_tok += (int64_t)tp * ph * pw;
    const int64_t T = P * ph * pw;
    const int32_t ring = 2 * (pw + 2) + 2 * ph;
    PS_REQUIRE(T < (int64_t)1 << 31 && P * ring < (int64_t)1 << 31, "pserve_plan: batch too large (%lld tokens)", (long long)T);

    pserve_plan_t* pl = new (std::nothrow) pserve_plan_t();
    if (!pl) { set_error("pserve_plan: out of host memory"); return PSERVE_ENOMEM; }
    struct Guard { pserve_plan_t* p; ~Guard() { delete p; } } guard{pl};

    // reorder requests by resolution: ascending (H, W), stable in arrival order
    std::vector<int32_t> perm(n);
    std::iota(perm.begin(), perm.end(), 0);
    std::stable_sort(perm.begin(), perm.end(), [&](int a, int b) {
        if (res[2 * a] != res[2 * b]) return res[2 * a] < res[2 * b];
        return res[2 * a + 1] < res[2 * b + 1];
    });
    pl->h_sorted_hw.resize(2 * n);
    int R = 0;
    for (int s = 0; s < n; ++s) {
        pl->h_sorted_hw[2 * s] = res[2 * perm[s]];
        pl->h_sorted_hw[2 * s + 1] = res[2 * perm[s] + 1];
        if (s == 0 || pl->h_sorted_hw[2 * s] != pl->h_sorted_hw[2 * s - 2] || pl->h_sorted_hw[2 * s + 1] != pl->h_sorted_hw[2 * s - 1]) ++R;
    }
    pl->n = n; pl->R = R; pl->P = (int32_t)P; pl->ph = ph; pl->pw = pw; pl->ring = ring; pl->T = T; pl->S = ph * pw;
    pl->max_tokens_per_image = (int32_t)max_tok;
    pl->text_len = text_len; pl->text_patches = tp;

    int64_t* cnt = pl->tab_count;
    cnt[PSERVE_TAB_PERM] = n;
    cnt[PSERVE_TAB_REQUEST_OFFSET] = n + 1;
    cnt[PSERVE_TAB_RES_OFFSET] = R + 1;
    cnt[PSERVE_TAB_RES_HW] = 2 * R;
    cnt[PSERVE_TAB_PATCH_OWNER] = P;
    cnt[PSERVE_TAB_PATCH_RC] = 2 * P;
    cnt[PSERVE_TAB_NEIGHBOUR] = 8 * P;
    cnt[PSERVE_TAB_HALO_SRC] = P * ring;
    cnt[PSERVE_TAB_CU_SEQLENS] = n + 1;
    cnt[PSERVE_TAB_SEQ_LEN] = n;
    for (int t = 0; t < PSERVE_TAB_COUNT; ++t) PS_TRY(pl->pool.alloc_t(&pl->d_tab[t], (size_t)cnt[t]));
    PS_TRY(pl->pool.alloc_t(&pl->d_sorted_hw, (size_t)2 * n));
    PS_TRY(pl->pool.alloc_t(&pl->mse_partial, (size_t)P * 16));

    hipStream_t st = (hipStream_t)stream;
    PS_CHECK_HIP(hipMemcpyAsync(pl->d_sorted_hw, pl->h_sorted_hw.data(), sizeof(int32_t) * 2 * n, hipMemcpyHostToDevice, st));
    PS_CHECK_HIP(hipMemcpyAsync(pl->d_tab[PSERVE_TAB_PERM], perm.data(), sizeof(int32_t) * n, hipMemcpyHostToDevice, st));
    plan_offsets_kernel<<<1, 1024, 0, st>>>(pl->d_sorted_hw, n, ph, pw, tp, text_len, pl->d_tab[PSERVE_TAB_REQUEST_OFFSET],
                                            pl->d_tab[PSERVE_TAB_CU_SEQLENS], pl->d_tab[PSERVE_TAB_RES_OFFSET],
                                            pl->d_tab[PSERVE_TAB_RES_HW], pl->d_tab[PSERVE_TAB_SEQ_LEN]);
    PS_TRY(check_launch("plan_offsets_kernel"));
    plan_patches_kernel<<<(unsigned)cdiv(P, 256), 256, 0, st>>>(pl->d_sorted_hw, pl->d_tab[PSERVE_TAB_REQUEST_OFFSET], n, (int32_t)P,
                                                      ph, pw, pl->d_tab[PSERVE_TAB_PATCH_OWNER], pl->d_tab[PSERVE_TAB_PATCH_RC],
                                                      pl->d_tab[PSERVE_TAB_NEIGHBOUR]);
    PS_TRY(check_launch("plan_patches_kernel"));
    plan_halo_kernel<<<(unsigned)cdiv(P * ring, 256), 256, 0, st>>>(pl->d_sorted_hw, pl->d_tab[PSERVE_TAB_REQUEST_OFFSET],
                                                          pl->d_tab[PSERVE_TAB_PATCH_OWNER], pl->d_tab[PSERVE_TAB_PATCH_RC],
                                                          (int32_t)P, ph, pw, ring, pl->d_tab[PSERVE_TAB_HALO_SRC]);
    PS_TRY(check_launch("plan_halo_kernel"));
    for (int t = 0; t < PSERVE_TAB_COUNT; ++t) {
        pl->h_tab[t].resize((size_t)cnt[t]);
        PS_CHECK_HIP(hipMemcpyAsync(pl->h_tab[t].data(), pl->d_tab[t], sizeof(int32_t) * cnt[t], hipMemcpyDeviceToHost, st));
    }
    PS_CHECK_HIP(hipStreamSynchronize(st));
    guard.p = nullptr;
    *out = pl;
    return PSERVE_OK;
}

int pserve_plan_text(const int32_t* res, int32_t n, int32_t ph, int32_t pw, int32_t text_len, void* stream,
                     pserve_plan_t** out) {
    return guarded("pserve_plan_text", [&] { return plan_text_impl(res, n, ph, pw, text_len, stream, out); });
}

void pserve_plan_free(pserve_plan_t* plan) { delete plan; }

int pserve_plan_info(const pserve_plan_t* plan, pserve_plan_info_t* out) {
    PS_REQUIRE(plan && out, "pserve_plan_info: NULL argument");
    out->n = plan->n; out->R = plan->R; out->P = plan->P; out->ph = plan->ph; out->pw = plan->pw;
    out->ring = plan->ring; out->T = plan->T;
    out->text_len = plan->text_len; out->text_patches = plan->text_patches;
    return PSERVE_OK;
}

int pserve_plan_table(const pserve_plan_t* plan, int which, int on_device, const int32_t** ptr, int64_t* count) {
    PS_REQUIRE(plan && ptr && count, "pserve_plan_table: NULL argument");
    PS_REQUIRE(which >= 0 && which < PSERVE_TAB_COUNT, "pserve_plan_table: unknown table %d", which);
    *ptr = on_device ? plan->d_tab[which] : plan->h_tab[which].data();
    *count = plan->tab_count[which];
    return PSERVE_OK;
}

int pserve_split(const pserve_plan_t* plan, const void* const* images, int32_t C, int dtype, void* x, void* stream) {
    return run_split<true>(plan, (void* const*)images, C, dtype, x, (hipStream_t)stream);
}

int pserve_reassemble(const pserve_plan_t* plan, const void* y, int32_t C, int dtype, void* const* images, void* stream) {
    return run_split<false>(plan, images, C, dtype, (void*)y, (hipStream_t)stream);
}

}  // extern "C"
